"""Host logic of bench.py that needs no GPU: the one-GPU contract, the algorithmic work the rooflines are
priced with, and the traffic records that are only valid for the kernel sources they were measured on."""
import json
import os
import subprocess
import sys
import types

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402
from workloads import get_workload  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_work_of_the_qwen3_shape():
    """4 H I flops per assignment in GEMM-1 (gate and up), 2 H I in GEMM-2; a resident expert's weights once
    per pass however many rows use it; gathered token rows and h per assignment."""
    wl = get_workload("qwen3_30b_a3b")
    H, I = wl.hidden, wl.inter
    counts = np.full(wl.n_slots, 256, dtype=np.int64)
    counts[3] = 0                                        # a resident expert nobody was routed to is not streamed
    w = bench.algorithmic_work(wl, counts, 0)
    A = 256 * (wl.n_slots - 1)
    assert w["assignments"] == A and w["active_slots"] == wl.n_slots - 1
    assert w["flops_gemm1"] == 4.0 * H * I * A and w["flops_gemm2"] == 2.0 * H * I * A
    assert w["flops_gate"] == 2.0 * wl.tokens * H * wl.n_experts
    assert w["bytes_gemm1"] == (wl.n_slots - 1) * 2 * I * H * 2 + A * H * 2 + A * I * 2
    assert w["bytes_gemm2"] == (wl.n_slots - 1) * I * H * 2 + A * I * 2 + A * H * 2
    assert w["bytes_layer_min"] == (wl.n_slots - 1) * 3 * I * H * 2 + wl.n_experts * H * 4 + 2 * wl.tokens * H * 2


def test_committed_traffic_records_match_the_sources():
    """Every record of profiles/traffic.json was taken on the kernel sources as they are now (otherwise the
    bench line would print traffic: null), and names its profile summary."""
    with open(bench.TRAFFIC_FILE) as f:
        rec = json.load(f)
    assert set(rec) == {"dsv3_ep8_rank", "qwen3_30b_a3b", "dsv3_ep8_decode"}
    for name, r in rec.items():
        assert bench.measured_traffic(name) == r["bytes_per_launch"] > 0, name
        assert r["bytes_per_launch"] == int((r["fetch_size_kib"] * r["fetch_scale"] + r["write_size_kib"] * r["write_scale"]) * 1024)
        assert os.path.exists(os.path.join(ROOT, r["profile"])), r["profile"]
    assert bench.measured_traffic("tiny_f32") is None    # no record: null, not a guess


def test_traffic_record_round_trip_and_staleness(tmp_path, monkeypatch):
    path = tmp_path / "traffic.json"
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(path))
    args = types.SimpleNamespace(record_traffic=["some_workload", "1000.5", "10", "2.0", "1.0"],
                                 traffic_kernel="k", traffic_profile="profiles/x.md")
    bench.record_traffic(args)
    assert bench.measured_traffic("some_workload") == int((1000.5 * 2.0 + 10 * 1.0) * 1024)
    rec = json.loads(path.read_text())
    assert rec["some_workload"]["kernel"] == "k" and rec["some_workload"]["sources"]
    # a record taken on other sources is not used
    rec["some_workload"]["source_sha256"] = "0" * 64
    path.write_text(json.dumps(rec))
    assert bench.measured_traffic("some_workload") is None
    # an unreadable file is no record either
    path.write_text("{")
    assert bench.measured_traffic("some_workload") is None
