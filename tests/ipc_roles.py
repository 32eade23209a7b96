"""The three processes of the zero-copy attach test (tests/test_gpu_ipc_attach.py), run as
`python tests/ipc_roles.py ROLE ...`:

  launcher  touches no GPU: starts the exporter, waits for its handles, starts the importer with them,
            tells the exporter to leave when the importer is done, exits with the importer's status.
  exporter  the memory owner: allocates the two weight pools, fills them with the seeded experts,
            exports their handles (one JSON line on stdout) and keeps them alive until told to leave.
  importer  a serving process: opens the handles, builds the layer over the ATTACHED pools (no weight
            is uploaded here), runs a forward through the C ABI and grades it against the CPU oracle.
"""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

SHAPE = dict(tokens=600, hidden=256, inter=128, n_experts=16, top_k=4, n_slots=17, n_local=12,
             act_dtype="bf16", router_dtype="bf16", gate="sigmoid_group", n_group=4, topk_group=2,
             routed_scale=2.5, n_shared=1, shared_range=(50, 500), seed=71)


def _workload():
    from workloads import MoEWorkload
    return MoEWorkload(name="ipc_attach", **SHAPE)


def _placement(wl):
    import numpy as np
    from workloads import block_expert_map, shared_slots_of
    slots = np.random.Generator(np.random.PCG64(9)).permutation(wl.n_slots - wl.n_shared)[:wl.n_local].astype(np.int32)
    return block_expert_map(wl.n_experts, 0, wl.n_local, slots), shared_slots_of(wl)


def launcher():
    me = os.path.abspath(__file__)
    exp = subprocess.Popen([sys.executable, "-u", me, "exporter"], stdin=subprocess.PIPE, stdout=subprocess.PIPE, text=True)
    try:
        line = exp.stdout.readline()
        if not line.startswith("{"):
            print("launcher: exporter did not deliver handles:", line, flush=True)
            return 3
        imp = subprocess.run([sys.executable, "-u", me, "importer", line.strip()], timeout=300)
        return imp.returncode
    finally:
        try:
            exp.stdin.write("leave\n")
            exp.stdin.flush()
        except OSError:
            pass
        try:
            exp.wait(timeout=60)
        except subprocess.TimeoutExpired:
            exp.kill()


def exporter():
    import torch
    from workloads import make_inputs, build_slot_pool
    from paper_2510_02613_amd.layer import export_pool, _dev
    wl = _workload()
    inp = make_inputs(wl)
    emap, shared = _placement(wl)
    dev = torch.device("cuda:0")
    w13 = _dev(build_slot_pool(inp["w13_experts"], emap, wl.n_slots, wl.n_local, shared), dev)
    w2 = _dev(build_slot_pool(inp["w2_experts"], emap, wl.n_slots, wl.n_local, shared), dev)
    torch.cuda.synchronize()
    h13, o13 = export_pool(w13)
    h2, o2 = export_pool(w2)
    print(json.dumps({"w13": [h13.hex(), o13], "w2": [h2.hex(), o2], "pid": os.getpid()}), flush=True)
    sys.stdin.readline()          # the pools stay allocated until the launcher says the importer is done
    torch.cuda.synchronize()


def importer(arg):
    import numpy as np
    import torch
    from gpu_util import Case, check_routing, check_bookkeeping, check_output, tensor_to_host
    from oracle import LayerSpec
    from workloads import make_inputs, build_slot_pool
    from paper_2510_02613_amd.layer import MoELayer, AttachedPool
    h = json.loads(arg)
    assert h["pid"] != os.getpid()
    wl = _workload()
    inp = make_inputs(wl)
    emap, shared = _placement(wl)
    elt = torch.int16
    free0, _ = torch.cuda.mem_get_info()
    p13 = AttachedPool(bytes.fromhex(h["w13"][0]), h["w13"][1], wl.n_slots, (2 * wl.inter, wl.hidden), elt)
    p2 = AttachedPool(bytes.fromhex(h["w2"][0]), h["w2"][1], wl.n_slots, (wl.hidden, wl.inter), elt)
    case = Case.__new__(Case)
    case.wl, case.inp, case.spec = wl, inp, LayerSpec.from_workload(wl)
    case.expert_map, case.shared_slots, case.select_bias = emap, shared, None
    # what the oracle is given: the pools as the EXPORTER built them (same seeded experts, same placement)
    case.w13_pool = build_slot_pool(inp["w13_experts"], emap, wl.n_slots, wl.n_local, shared)
    case.w2_pool = build_slot_pool(inp["w2_experts"], emap, wl.n_slots, wl.n_local, shared)
    # the attached memory holds exactly that, and this process never wrote it
    used = sorted(set(int(s) for s in emap if s >= 0) | set(int(s) for s in shared))
    for s in used:
        np.testing.assert_array_equal(tensor_to_host(p13.tensor[s]), case.w13_pool[s])
        np.testing.assert_array_equal(tensor_to_host(p2.tensor[s]), case.w2_pool[s])
    case.layer = MoELayer(hidden=wl.hidden, inter=wl.inter, n_experts=wl.n_experts, top_k=wl.top_k, n_slots=wl.n_slots,
                          max_tokens=wl.tokens, act_dtype=wl.act_dtype, router_dtype=wl.router_dtype, gate=wl.gate,
                          n_group=wl.n_group, topk_group=wl.topk_group, renormalize=wl.renormalize,
                          routed_scale=wl.routed_scale, n_shared=wl.n_shared, router_w=inp["router_w"],
                          logit_bias=inp["logit_bias"], w13_pool=p13, w2_pool=p2)
    assert case.layer.w13.data_ptr() == p13.ptr and case.layer.w2.data_ptr() == p2.ptr
    case.layer.set_expert_map(emap, shared)
    case.x_dev = case.layer.upload(inp["x"])
    out = case.run()
    v = case.layer.view(wl.tokens)
    ids, _, _ = check_routing(case, v["topk_ids"], v["topk_w"])
    check_bookkeeping(case, v, wl.tokens, wl.shared_range)
    err = check_output(case, out, ids)
    case.layer.close()
    p13.close()
    p2.close()
    print(f"importer: attached pools {p13.n_vslots} slots, forward max rel err {err:.2e} OK", flush=True)


if __name__ == "__main__":
    role = sys.argv[1]
    if role == "launcher":
        sys.exit(launcher())
    if role == "exporter":
        exporter()
    elif role == "importer":
        importer(sys.argv[2])
    else:
        sys.exit(f"unknown role {role}")
