#!/usr/bin/env python3
"""Benchmark of the MoE rank layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload all|NAME]

A step is one whole forward pass of the layer (gate, permute, both grouped expert
GEMMs, combine) over one batch of synthetic tokens that is already resident in
HBM.  By default all five benchmark configurations run, one after the other, in
this process; the headline (`value`, `config.workload`, `roofline`,
`cpu_baseline`) is the largest one, the DeepSeek-V3-shaped rank, and `workloads`
carries the same figures for every configuration: step time, tokens/s, per-kernel
times, the roofline position of the dominant kernel (timed with HIP events on the
pass's own stream, inside the timed region) and of the whole layer -- against the
bf16 MFMA peak for the prefill-sized batches, against the HBM peak for the
decode-sized one -- and, for the re-layout configuration, both phases, the
slot-order placement and what the switches did to device memory.  The fp64 CPU
oracle is timed on a bounded token sample of the headline workload on this machine's
host cores.  Prints ONE JSON line.

Only one GPU is used: the layer is one expert-parallel rank's share of the work.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# published MI355X peaks
PEAK_BF16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0
PEAK_F32_VALU_TFLOPS = 157.3

# the five benchmark configurations, headline first
HEADLINE = "dsv3_ep8_rank"
ALL_WORKLOADS = ("dsv3_ep8_rank", "qwen3_30b_a3b", "dsv3_ep8_decode", "qwen3_relayout", "tiny_f32")

# HBM traffic of the dominant kernel per launch, measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE,
# each scaled by what the same counter reads for a plain copy of known size).  The record names the
# kernel and carries a hash of the sources it was taken on: when those have changed since, the figure
# is stale and `traffic` is null.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")


def source_hash(paths):
    h = hashlib.sha256()
    for rel in sorted(paths):
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(rel.encode() + b"\0" + f.read() + b"\0")
    return h.hexdigest()


def measured_traffic(workload):
    """Bytes per launch of the dominant kernel from profiles/traffic.json, or None when there is no record
    for this workload or the kernel's sources have changed since it was taken."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f).get(workload)
        if not rec or source_hash(rec["sources"]) != rec["source_sha256"]:
            return None
        return int(rec["bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        return None


def record_traffic(args):
    """--record-traffic WORKLOAD FETCH_KIB WRITE_KIB FETCH_SCALE WRITE_SCALE: store the counter figures of a
    rocprofv3 --pmc run (KiB per launch of the dominant kernel, summed over its launches of one pass) with
    the hash of the kernel sources as they are now."""
    name, fetch_kib, write_kib, fs, ws_ = args.record_traffic
    sources = sorted(os.path.join("paper_2510_02613_amd", "csrc", f)
                     for f in os.listdir(os.path.join(ROOT, "paper_2510_02613_amd", "csrc"))
                     if f.startswith("k_experts") or f in ("moe_internal.h", "k_permute.hip"))
    try:
        with open(TRAFFIC_FILE) as f:
            allrec = json.load(f)
    except OSError:
        allrec = {}
    allrec[name] = {
        "kernel": args.traffic_kernel, "profile": args.traffic_profile,
        "fetch_size_kib": float(fetch_kib), "write_size_kib": float(write_kib),
        "fetch_scale": float(fs), "write_scale": float(ws_),
        "bytes_per_launch": int((float(fetch_kib) * float(fs) + float(write_kib) * float(ws_)) * 1024),
        "sources": sources, "source_sha256": source_hash(sources),
    }
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(allrec, f, indent=1, sort_keys=True)
        f.write("\n")
    print(json.dumps(allrec[name]))


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="all",
                    help="all (the five configurations, headline dsv3_ep8_rank) | dsv3_ep8_rank | qwen3_30b_a3b | "
                         "dsv3_ep8_decode | qwen3_relayout | tiny_f32 | dsv2_lite")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-phase-events", action="store_true",
                    help="do not record per-kernel events inside the timed region (roofline then is null)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--scale-while-serve", type=int, default=None, metavar="BLOCKS",
                    help="qwen3_relayout only: after the timed region also time the phase-A layer idle, then with the 32 "
                         "new experts being filled into free slots on a side stream by copy kernels of BLOCKS workgroups, "
                         "then the phase-B layer after the switch")
    ap.add_argument("--replicate-hot", type=int, default=None, metavar="N",
                    help="qwen3_relayout only: after the timed region also time the phase-A layer (32 experts resident, "
                         "Zipf-skewed routing) with plain placement and with the N most loaded experts copied into spare slots")
    ap.add_argument("--hip-graph", action="store_true",
                    help="capture one forward into a HIP graph and time replays of it (no per-kernel events, so no roofline)")
    ap.add_argument("--virtual-pool", action="store_true",
                    help="back the two weight pools with contiguous virtual tensors over separately allocated physical "
                         "pages (moe_vpool_*), pages mapped in a shuffled order, instead of plain allocations")
    ap.add_argument("--flags", type=int, default=0, help="MOE_FLAG_* bits passed to every forward (testing aids of the library)")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the two measuring-stick kernels (sustained MFMA rate, streaming read) after the timed region")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a 1 GiB device copy (counter calibration for rocprofv3 --pmc) and exit")
    ap.add_argument("--record-traffic", nargs=5, metavar=("WORKLOAD", "FETCH_KIB", "WRITE_KIB", "FETCH_SCALE", "WRITE_SCALE"),
                    help="no GPU work: store counter figures of a rocprofv3 --pmc run in profiles/traffic.json")
    ap.add_argument("--traffic-kernel", default="grouped GEMM-1 + SwiGLU", help="with --record-traffic: kernel symbol(s) the figures are for")
    ap.add_argument("--traffic-profile", default="", help="with --record-traffic: the profiles/ summary that holds the command and the raw figures")
    return ap.parse_args()


def algorithmic_work(wl, counts, shared_rows):
    """Useful flops and minimum HBM bytes of one pass (no padding rows, every needed byte once)."""
    H, I, E, T = wl.hidden, wl.inter, wl.n_experts, wl.tokens
    es = 2 if wl.act_dtype == "bf16" else 4
    rs = 2 if wl.router_dtype == "bf16" else 4
    A = int(counts.sum())
    active = int((counts > 0).sum())
    flops_gemm1 = 4.0 * H * I * A
    flops_gemm2 = 2.0 * H * I * A
    flops_gate = 2.0 * T * H * E
    bytes_w13 = active * 2 * I * H * es
    bytes_w2 = active * H * I * es
    return {
        "assignments": A, "active_slots": active,
        "flops_gemm1": flops_gemm1, "flops_gemm2": flops_gemm2, "flops_gate": flops_gate,
        "flops_total": flops_gemm1 + flops_gemm2 + flops_gate,
        # GEMM-1 reads its weights once, gathers each token row once per assignment, writes h
        "bytes_gemm1": bytes_w13 + A * H * es + A * I * es,
        "bytes_gemm2": bytes_w2 + A * I * es + A * H * es,
        # whole layer minimum: weights + router + x in + out
        "bytes_layer_min": bytes_w13 + bytes_w2 + E * H * rs + 2 * T * H * es,
    }


def run_workload(torch, args, name, extras=False):
    """Builds the layer of one configuration on the GPU, times args.steps passes after args.warmup, and
    returns (figures for the JSON line, state for the optional legs that follow)."""
    from workloads import get_workload, make_inputs, relayout_maps, block_expert_map, shared_slots_of, build_slot_pool
    from paper_2510_02613_amd import binding as B
    from paper_2510_02613_amd.layer import MoELayer
    dev = torch.device("cuda:0")
    wl = get_workload(name)
    inp = make_inputs(wl, threads=16)
    if wl.name == "qwen3_relayout":
        expert_map = relayout_maps(wl)[1]
    else:
        expert_map = block_expert_map(wl.n_experts, 0, wl.n_local)
    shared = shared_slots_of(wl)
    pools = {}
    if args.virtual_pool:
        from paper_2510_02613_amd.layer import VirtualPool
        elt = torch.int16 if wl.act_dtype == "bf16" else torch.float32
        pools = {"w13_pool": VirtualPool(wl.n_slots, (2 * wl.inter, wl.hidden), elt, dev),
                 "w2_pool": VirtualPool(wl.n_slots, (wl.hidden, wl.inter), elt, dev)}
        order = np.random.Generator(np.random.PCG64(7)).permutation(wl.n_slots)
        for pool in pools.values():
            pages = [pool.page_alloc() for _ in range(wl.n_slots)]
            for s in range(wl.n_slots):
                pool.map(s, pages[int(order[s])])
    layer = MoELayer(hidden=wl.hidden, inter=wl.inter, n_experts=wl.n_experts, top_k=wl.top_k,
                     n_slots=wl.n_slots, max_tokens=wl.tokens, act_dtype=wl.act_dtype,
                     router_dtype=wl.router_dtype, gate=wl.gate, n_group=wl.n_group,
                     topk_group=wl.topk_group, renormalize=wl.renormalize, routed_scale=wl.routed_scale,
                     n_shared=wl.n_shared, router_w=inp["router_w"], logit_bias=inp["logit_bias"], device=dev, **pools)
    w13_pool = build_slot_pool(inp["w13_experts"], expert_map, wl.n_slots, wl.n_local, shared)
    w2_pool = build_slot_pool(inp["w2_experts"], expert_map, wl.n_slots, wl.n_local, shared)
    layer.load_pool(w13_pool, w2_pool)
    layer.set_expert_map(expert_map, shared if wl.n_shared else None)
    x = layer.upload(inp["x"])
    out = torch.empty_like(x)
    stream = torch.cuda.current_stream(dev)

    def step():
        layer.forward(x, out=out, shared_range=wl.shared_range, stream=stream, flags=args.flags)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.hip_graph:
        side = torch.cuda.Stream(device=dev)
        with torch.cuda.stream(side):
            layer.forward(x, out=out, shared_range=wl.shared_range, stream=side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            layer.forward(x, out=out, shared_range=wl.shared_range, stream=side)
        step = graph.replay
        for _ in range(3):
            step()
        torch.cuda.synchronize()
    use_events = not args.no_phase_events and not args.hip_graph
    # Inside the timed region only the dominant kernel (GEMM-1) is bracketed by events, on every 4th step: each
    # record costs the stream a microsecond or two, and six per step would be 1.5 % (prefill) to 3.5 % (decode) of
    # the step itself.  The other phases are timed on 8 further steps after the timed region.
    every = 4 if args.steps >= 8 else 1
    GEMM1 = B.PHASE_NAMES.index("gemm1")
    if use_events:
        B.moe_profile_enable(layer.handle, 1)
        step()  # events exist now; keep their first use out of the timed region
        torch.cuda.synchronize()
        B.moe_profile_select(layer.handle, GEMM1)
        B.moe_profile_enable(layer.handle, every)

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    phases = None
    if use_events:
        n = min((args.steps + every - 1) // every, 64)   # recorded steps of the timed region
        gemm1_ms = sum(B.moe_profile_read(layer.handle, back)[GEMM1] for back in range(n)) / n
        B.moe_profile_select(layer.handle, -1)           # all phases, every step, outside the timed region
        B.moe_profile_enable(layer.handle, 1)
        n_extra = 8
        for _ in range(n_extra):
            step()
        torch.cuda.synchronize()
        acc = np.zeros(B.MOE_N_PHASES)
        for back in range(n_extra):
            acc += np.array(B.moe_profile_read(layer.handle, back))
        phases = dict(zip(B.PHASE_NAMES, (acc / n_extra).tolist()))
        phases["gemm1"] = gemm1_ms                       # the dominant kernel: from the timed region
        B.moe_profile_enable(layer.handle, 0)

    view = layer.view(wl.tokens)
    counts = view["counts"]
    work = algorithmic_work(wl, counts, wl.shared_range[1] - wl.shared_range[0])
    decode = wl.name == "dsv3_ep8_decode"
    t_step = ms_per_step * 1e-3

    # whole layer against both roofs; the one the metric names for this batch size is `bound`
    layer_fig = {"bound": "hbm" if decode else "mfma",
                 "tflops": work["flops_total"] / t_step / 1e12,
                 "frac_bf16_mfma_peak": work["flops_total"] / t_step / 1e12 / PEAK_BF16_MFMA_TFLOPS,
                 "min_hbm_gbs": work["bytes_layer_min"] / t_step / 1e9,
                 "frac_hbm_peak": work["bytes_layer_min"] / t_step / 1e9 / PEAK_HBM_GBS,
                 "phase_us": {k: v * 1e3 for k, v in phases.items()} if phases else None,
                 "phase_us_source": "gemm1: HIP events on every 4th step of the timed region; the other phases: events on 8 steps run after it"}
    if wl.act_dtype != "bf16":
        layer_fig["bound"] = "launch latency (fp32 parity configuration: 6 MFLOP per pass)"

    roofline = None
    if phases and wl.act_dtype == "bf16":
        dom = "gemm1"
        t_dom = phases[dom] * 1e-3
        gbs = work["bytes_gemm1"] / t_dom / 1e9
        tfl = work["flops_gemm1"] / t_dom / 1e12
        hbm = {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS}
        mfma = {"bound": "mfma", "achieved": tfl, "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": tfl / PEAK_BF16_MFMA_TFLOPS}
        roofline = dict(hbm if decode else mfma)
        roofline["kernel"] = "grouped GEMM-1 + SwiGLU"
        # the same launch against the other roof: with ~256 rows per expert the prefill kernel sits below the
        # ridge (flops per algorithmic byte < 2500/8), so HBM is the tighter of its two roofs
        roofline["other_roof"] = dict(mfma if decode else hbm, flop_per_byte=work["flops_gemm1"] / work["bytes_gemm1"],
                                      ridge_flop_per_byte=PEAK_BF16_MFMA_TFLOPS * 1e3 / PEAK_HBM_GBS)
        roofline["traffic"] = measured_traffic(wl.name)
        roofline["avg_launch_us"] = phases[dom] * 1e3
        roofline["algorithmic_per_launch"] = work["bytes_gemm1"] if decode else work["flops_gemm1"]
        roofline["layer_frac"] = layer_fig["frac_hbm_peak"] if decode else layer_fig["frac_bf16_mfma_peak"]

    fig = {
        "ms_per_step": ms_per_step, "tokens_per_s": wl.tokens / t_step, "dtype": wl.act_dtype,
        "config": {"workload": wl.name, "weight_pools": "virtual (moe_vpool)" if args.virtual_pool else "plain",
                   "launch": "hip graph replay" if args.hip_graph else "eager", "tokens": wl.tokens, "hidden": wl.hidden, "inter": wl.inter,
                   "n_experts": wl.n_experts, "top_k": wl.top_k, "local_slots": int((expert_map >= 0).sum()) + wl.n_shared,
                   "gate": wl.gate, "assignments": work["assignments"], "active_slots": work["active_slots"],
                   "rows_per_slot_max": int(counts.max()), "rows_per_slot_mean": float(counts[counts > 0].mean()) if (counts > 0).any() else 0.0},
        "layer": layer_fig, "roofline": roofline,
    }
    state = dict(wl=wl, inp=inp, layer=layer, x=x, out=out, stream=stream, w13_pool=w13_pool, w2_pool=w2_pool,
                 expert_map=expert_map, shared=shared, pools=pools)
    if wl.name == "qwen3_relayout":
        fig["relayout"] = relayout_report(torch, layer, wl, inp, x, out, stream, w13_pool, w2_pool)
    return fig, state


def release(torch, state):
    torch.cuda.synchronize()
    state["layer"].close()
    for pool in state["pools"].values():
        pool.close()
    state.clear()
    torch.cuda.empty_cache()


def main():
    args = parse_args()
    if args.record_traffic:
        record_traffic(args)
        return
    if args.gpus != 1:
        print("bench.py: this build runs one expert-parallel rank on ONE GPU; --gpus must be 1 "
              "(no collectives or sharding are part of it)", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")

    if args.copy_calibration:
        n = 1 << 30
        src = torch.empty(n, dtype=torch.uint8, device=dev).zero_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_each_way": n, "launches": 5}))
        return

    from paper_2510_02613_amd import binding as B
    names = ALL_WORKLOADS if args.workload == "all" else (args.workload,)
    single = len(names) == 1
    for flag, val in (("--scale-while-serve", args.scale_while_serve), ("--replicate-hot", args.replicate_hot)):
        if val is not None and names != ("qwen3_relayout",):
            print(f"bench.py: {flag} needs --workload qwen3_relayout", file=sys.stderr)
            sys.exit(2)

    head_fig, extras, per_workload = None, {}, {}
    for i, name in enumerate(names):
        t_wall = time.perf_counter()
        fig, state = run_workload(torch, args, name)
        if i == 0:
            head_fig = fig
            wl = state["wl"]
            if args.scale_while_serve is not None:
                extras["scale_while_serve"] = scale_while_serve(torch, state["layer"], wl, state["inp"], state["x"], state["out"], state["stream"], args)
            if args.replicate_hot is not None:
                if not 0 < args.replicate_hot <= wl.n_slots // 2:
                    print("bench.py: --replicate-hot N needs 0 < N <= %d" % (wl.n_slots // 2), file=sys.stderr)
                    sys.exit(2)
                extras["replicate_hot"] = replicate_hot(torch, state["layer"], wl, state["x"], state["out"], state["stream"], args.replicate_hot)
            if not args.no_ceilings:
                extras["ceilings"] = measure_ceilings(torch, B, state["layer"], state["stream"])
            if not args.no_cpu_baseline:
                extras["cpu_baseline"] = cpu_baseline(wl, state["inp"], state["w13_pool"], state["w2_pool"], state["expert_map"],
                                                      state["shared"], args.cpu_seconds)
        fig["wall_s"] = time.perf_counter() - t_wall
        per_workload[name] = fig
        print(f"bench.py: {name}: {fig['ms_per_step'] * 1e3:.1f} us/step", file=sys.stderr, flush=True)
        release(torch, state)

    result = {
        "metric": "MoE layer tokens/s at 1 MI355X; % bf16 MFMA peak (prefill), % HBM BW (decode)",
        "value": head_fig["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head_fig["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head_fig["dtype"], "data": "synthetic",
        "config": head_fig["config"], "layer": head_fig["layer"], "roofline": head_fig["roofline"],
    }
    if "relayout" in head_fig:
        result["relayout"] = head_fig["relayout"]
    result.update(extras)
    if not single:
        result["workloads"] = {n: {k: v for k, v in f.items() if k != "dtype"} for n, f in per_workload.items()}
    print(json.dumps(result))


def scale_while_serve(torch, layer, wl, inp, x, out, stream, args):
    """Forward time of the phase-A layer (32 experts resident), the same while the other 32 experts are
    copied into free slots on a side stream, and of the phase-B layer after the map switch."""
    from workloads import relayout_maps
    map_a, map_b = relayout_maps(wl)
    copy = torch.cuda.Stream(device=x.device)
    new = list(range(wl.n_slots // 2, wl.n_slots))
    src = [(layer.upload(inp["w13_experts"][e]), layer.upload(inp["w2_experts"][e])) for e in new]
    nbytes = sum(a.numel() * a.element_size() + b.numel() * b.element_size() for a, b in src)
    layer.set_expert_map(map_a)

    c0, c1, w0, w1 = (torch.cuda.Event(enable_timing=True) for _ in range(4))

    def timed(n, fill):
        for _ in range(3):
            layer.forward(x, out=out, shared_range=wl.shared_range, stream=stream)
        torch.cuda.synchronize()
        if fill:
            # The whole set of new experts, enqueued first (this host thread needs ~0.1 ms per fill, and a
            # serving loop that stops to issue them would be what is measured); the copies run on their
            # stream while the forwards below are enqueued and run.
            c0.record(copy)
            for j, e in enumerate(new):
                layer.load_expert_async(int(map_b[e]), src[j][0], src[j][1], copy, stream, copy_blocks=args.scale_while_serve)
            c1.record(copy)
        w0.record(stream)
        for i in range(n):
            layer.forward(x, out=out, shared_range=wl.shared_range, stream=stream)
        w1.record(stream)
        torch.cuda.synchronize()
        return w0.elapsed_time(w1) / n

    n = 16
    idle = timed(n, False)
    busy = timed(n, True)
    fill_ms = c0.elapsed_time(c1)
    overlap_ms = max(0.0, min(w0.elapsed_time(c1), w0.elapsed_time(w1)))   # part of the forwards' window with copies running
    layer.set_expert_map(map_b)              # waits (on the stream) for the fills
    after = timed(n, False)
    return {"copy_blocks": args.scale_while_serve, "forwards": n,
            "ms_per_step_phase_a_idle": idle, "ms_per_step_phase_a_beside_fill": busy,
            "window_ms": busy * n, "window_ms_with_copies_running": overlap_ms,
            "fill_bytes": nbytes, "fill_ms": fill_ms, "fill_gbs": nbytes / (fill_ms * 1e-3) / 1e9,
            "ms_per_step_phase_b_after_switch": after}


def relayout_report(torch, layer, wl, inp, x, out, stream, w13_pool_b, w2_pool_b):
    """The re-layout workload on its three placements, 16 forwards each after 3 warm-ups: phase A (experts
    0..31 resident), phase B (64 resident, the new 32 in shuffled slots: the placement the timed region ran
    on), and phase B with the new experts in slot order (what a freshly built contiguous layout would be).
    Also what the switches changed: nothing but the table (pool and workspace addresses, free device memory)."""
    from workloads import relayout_maps, build_slot_pool
    map_a, map_b = relayout_maps(wl)
    half = wl.n_slots // 2
    map_c = map_b.copy()
    map_c[half:2 * half] = np.arange(half, 2 * half, dtype=np.int32)     # contiguous: expert e in slot e
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ptrs = (layer.w13.data_ptr(), layer.w2.data_ptr(), layer.workspace.data_ptr())
    free0, _ = torch.cuda.mem_get_info()

    def timed(n=16):
        for _ in range(3):
            layer.forward(x, out=out, shared_range=wl.shared_range, stream=stream)
        e0.record(stream)
        for _ in range(n):
            layer.forward(x, out=out, shared_range=wl.shared_range, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / n
        counts = layer.view(wl.tokens)["counts"]
        work = algorithmic_work(wl, counts, 0)
        return {"ms_per_step": ms, "assignments": work["assignments"], "active_slots": work["active_slots"],
                "assignments_per_s": work["assignments"] / (ms * 1e-3),
                "tflops": work["flops_total"] / (ms * 1e-3) / 1e12,
                "min_hbm_gbs": work["bytes_layer_min"] / (ms * 1e-3) / 1e9}

    rep = {}
    layer.set_expert_map(map_a)                       # the weights of phase B's pool hold phase A's experts in place
    rep["phase_a_32_experts"] = timed()
    layer.set_expert_map(map_b)
    first_b = timed()
    out_b = out.clone()
    free1, _ = torch.cuda.mem_get_info()              # before the slot-order pool is staged for the comparison
    same = ptrs == (layer.w13.data_ptr(), layer.w2.data_ptr(), layer.workspace.data_ptr())
    # the two phase-B placements alternate three times (device-side pool copies), so that drift of the
    # box between the measurements is not read as a difference between them
    pool_b = (layer.w13.clone(), layer.w2.clone())
    pool_c = (layer.upload(build_slot_pool(inp["w13_experts"], map_c, wl.n_slots, wl.n_local, ())),
              layer.upload(build_slot_pool(inp["w2_experts"], map_c, wl.n_slots, wl.n_local, ())))
    runs_b, runs_c = [first_b], []
    identical = True
    for rnd in range(3):
        layer.w13.copy_(pool_c[0]); layer.w2.copy_(pool_c[1])
        layer.set_expert_map(map_c)
        runs_c.append(timed())
        identical = identical and bool(torch.equal(out_b, out))
        layer.w13.copy_(pool_b[0]); layer.w2.copy_(pool_b[1])
        layer.set_expert_map(map_b)                   # ends on the placement of the timed region
        if rnd < 2:
            runs_b.append(timed())

    def mean(runs):
        m = dict(runs[0])
        for key in ("ms_per_step", "assignments_per_s", "tflops", "min_hbm_gbs"):
            m[key] = float(np.mean([r[key] for r in runs]))
        m["ms_per_step_runs"] = [r["ms_per_step"] for r in runs]
        return m

    rep["phase_b_64_experts_shuffled_slots"] = mean(runs_b)
    rep["phase_b_64_experts_slot_order"] = mean(runs_c)
    rep["outputs_identical_shuffled_vs_slot_order"] = identical
    rep["pool_and_workspace_addresses_unchanged"] = bool(same)
    rep["device_memory_taken_by_the_switches_bytes"] = int(free0 - free1)
    torch.cuda.synchronize()
    return rep


def replicate_hot(torch, layer, wl, x, out, stream, n_hot):
    """Forward time of the phase-A layer (experts 0..31 in slots 0..31, the other slots spare) with the
    plain placement and with a second copy of each of the n_hot most loaded experts in a spare slot."""
    from workloads import relayout_maps
    map_a, _ = relayout_maps(wl)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(n=16):
        for _ in range(3):
            layer.forward(x, out=out, shared_range=wl.shared_range, stream=stream)
        e0.record(stream)
        for _ in range(n):
            layer.forward(x, out=out, shared_range=wl.shared_range, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    layer.set_expert_map(map_a)
    plain = timed()
    counts = layer.view(x.shape[0])["counts"]
    local = [e for e in range(wl.n_experts) if map_a[e] >= 0]
    hot = sorted(local, key=lambda e: -int(counts[map_a[e]]))[:n_hot]
    spare = [s for s in range(wl.n_slots) if s not in set(int(v) for v in map_a if v >= 0)]
    replicas = [[int(map_a[e])] if map_a[e] >= 0 else [] for e in range(wl.n_experts)]
    with torch.cuda.stream(stream):
        for e in hot:
            s = spare.pop()
            layer.w13[s].copy_(layer.w13[int(map_a[e])])
            layer.w2[s].copy_(layer.w2[int(map_a[e])])
            replicas[e].append(s)
    layer.set_expert_replicas(replicas, stream=stream)
    rep = timed()
    counts_rep = layer.view(x.shape[0])["counts"]
    return {"copies": n_hot, "ms_per_step_plain": plain, "ms_per_step_replicated": rep,
            "largest_group_rows_plain": int(counts.max()), "largest_group_rows_replicated": int(counts_rep.max()),
            "slots_in_use_plain": int((counts > 0).sum()), "slots_in_use_replicated": int((counts_rep > 0).sum())}


def measure_ceilings(torch, B, layer, stream):
    """What this chip sustains with nothing else in the way (after the timed region, same process):
    a register-only bf16 MFMA stream shaped like the expert kernels' wavefronts, and one plain
    streaming read of the layer's own W13 pool.  Context for the roofline fractions, which are
    taken against the data-sheet peaks."""
    sink = torch.zeros(1, dtype=torch.float32, device=layer.w13.device)
    s = stream.cuda_stream
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
    w_ptr, w_bytes = layer.w13.data_ptr(), layer.w13.numel() * layer.w13.element_size()
    B.moe_ceiling_mfma(512, 2000, False, sink.data_ptr(), s)          # warm all three
    B.moe_ceiling_mfma(512, 2000, True, sink.data_ptr(), s)
    B.moe_ceiling_stream(w_ptr, w_bytes, sink.data_ptr(), s)
    ev[0].record(stream)
    flops = B.moe_ceiling_mfma(2048, 20000, False, sink.data_ptr(), s)   # tens of ms each
    ev[1].record(stream)
    B.moe_ceiling_mfma(2048, 20000, True, sink.data_ptr(), s)
    ev[2].record(stream)
    reps = max(1, int(8e9 // w_bytes))
    for _ in range(reps):
        B.moe_ceiling_stream(w_ptr, w_bytes, sink.data_ptr(), s)
    ev[3].record(stream)
    # the same pool read in the access shape of the large-tile kernels' weight loaders (bf16 pools with whole 128-byte steps)
    S, rows, H = layer.w13.shape
    row_bytes = H * layer.w13.element_size()
    tiles = S * (rows // 256)
    shaped = layer.act_dtype == "bf16" and row_bytes % 128 == 0 and tiles > 0 and rows % 256 == 0
    if shaped:
        for nt in (False, True):
            B.moe_ceiling_tile_stream(w_ptr, tiles, row_bytes, nt, s)    # warm
        for i, nt in enumerate((False, True)):
            for _ in range(reps):
                B.moe_ceiling_tile_stream(w_ptr, tiles, row_bytes, nt, s)
            ev[4 + i].record(stream)
    torch.cuda.synchronize()
    t_c = ev[0].elapsed_time(ev[1]) * 1e-3
    t_r = ev[1].elapsed_time(ev[2]) * 1e-3
    t_s = ev[2].elapsed_time(ev[3]) * 1e-3
    out = {"mfma_bf16_tflops_constant_operands": flops / t_c / 1e12,
           "mfma_bf16_tflops_random_operands": flops / t_r / 1e12,
           "stream_read_gbs": reps * w_bytes / t_s / 1e9, "stream_bytes": w_bytes, "stream_reps": reps,
           "note": "sustained rates of this chip: register-only v_mfma_f32_32x32x16_bf16 (8 wavefronts per workgroup) "
                   "on constant and on changing pseudo-random operands, a plain read of the W13 pool, and the same pool "
                   "read as the large-tile kernels' weight loaders read it (256-row tiles, 128 bytes per row per step, "
                   "global -> LDS, default and non-temporal)"}
    if shaped:
        out["tile_stream_read_gbs"] = reps * w_bytes / (ev[3].elapsed_time(ev[4]) * 1e-3) / 1e9
        out["tile_stream_read_nt_gbs"] = reps * w_bytes / (ev[4].elapsed_time(ev[5]) * 1e-3) / 1e9
    return out


def cpu_baseline(wl, inp, w13_pool, w2_pool, expert_map, shared, target_s):
    """The fp64 oracle, as it stands, on a bounded random token sample of the same workload."""
    import oracle
    from oracle import LayerSpec
    spec = LayerSpec.from_workload(wl)
    g = np.random.Generator(np.random.PCG64(99))

    def run(n):
        tok = np.sort(g.choice(wl.tokens, size=n, replace=False)).astype(np.int32)
        t0 = time.perf_counter()
        oracle.forward(spec, inp["x"], inp["router_w"], w13_pool, w2_pool, expert_map,
                       logit_bias=inp["logit_bias"], shared_slots=shared, shared_range=wl.shared_range, tokens=tok)
        return time.perf_counter() - t0

    threads = oracle.max_threads()
    n0 = min(wl.tokens, 8 * threads)   # a probe of two tokens per thread overestimates the time per token by half
    t_probe = run(n0)
    n = int(max(n0, min(wl.tokens, n0 * target_s / max(t_probe, 1e-3))))
    n = max(threads, n // threads * threads) if n < wl.tokens else wl.tokens
    t = run(n)
    return {"value": n / t, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"{n} of {wl.tokens} tokens (random, all their local assignments), fp64, "
                      f"{t:.1f} s wall; probe {n0} tokens {t_probe:.2f} s"}


if __name__ == "__main__":
    main()
