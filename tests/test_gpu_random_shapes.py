"""Seeded random layer shapes through every dispatch boundary (contraction lengths that are and are not
whole K-steps, batches on both sides of the kernel-family thresholds, both gates, remote experts, shared
experts, sparse slot pools), each checked in full against the oracle."""
import numpy as np
import pytest

from workloads import MoEWorkload

pytestmark = pytest.mark.gpu


def _random_case(i):
    g = np.random.Generator(np.random.PCG64(1000 + i))
    pick = lambda xs: xs[int(g.integers(len(xs)))]
    act = pick(["bf16", "bf16", "bf16", "f32"])
    hidden = int(pick([64, 72, 128, 136, 192, 256, 264, 320, 512]))
    inter = int(pick([8, 64, 72, 128, 136, 192, 264]))
    gate = pick(["softmax", "sigmoid_group"])
    if gate == "sigmoid_group":
        n_group = int(pick([2, 4, 8]))
        per = int(pick([2, 4, 8, 16]))
        n_experts = n_group * per
        topk_group = int(g.integers(1, n_group + 1))
        top_k = int(g.integers(1, min(8, topk_group * per) + 1))
    else:
        n_group, topk_group = 1, 1
        n_experts = int(pick([4, 8, 24, 40, 64, 96, 130]))
        top_k = int(g.integers(1, min(8, n_experts) + 1))
    n_shared = int(pick([0, 0, 1, 2]))
    n_local = int(g.integers(1, n_experts + 1))
    spare = int(pick([0, 0, 3]))
    n_slots = n_local + n_shared + spare
    tokens = int(pick([1, 2, 5, 17, 40, 130, 257, 600, 1500, 2600]))
    b = int(g.integers(0, tokens + 1))
    e = int(g.integers(b, tokens + 1))
    wl = MoEWorkload(name=f"rand{i}", tokens=tokens, hidden=hidden, inter=inter, n_experts=n_experts, top_k=top_k,
                     n_slots=n_slots, n_local=n_local, act_dtype=act, router_dtype=pick(["f32", "bf16"]) if act == "bf16" else "f32",
                     gate=gate, n_group=n_group, topk_group=topk_group, renormalize=bool(g.integers(2)),
                     routed_scale=float(pick([1.0, 2.5])), n_shared=n_shared, shared_range=(b, e) if n_shared else (0, 0),
                     zipf_s=float(pick([0.0, 0.0, 1.2])), seed=2000 + i)
    # which logical experts are local, and in which (scattered) slots
    local = np.sort(g.choice(n_experts, size=n_local, replace=False))
    slots = g.permutation(n_local + spare)[:n_local]
    emap = np.full(n_experts, -1, np.int32)
    emap[local] = slots
    return wl, emap, local


def _random_large_case(i):
    """Prefill-sized bf16 layers: long contractions (with and without a split last round), contraction
    lengths that the large-tile kernels take and do not take, many rows per slot."""
    g = np.random.Generator(np.random.PCG64(5000 + i))
    pick = lambda xs: xs[int(g.integers(len(xs)))]
    hidden = int(pick([512, 1024, 2048, 4096, 4160, 7168]))
    inter = int(pick([64, 128, 192, 320, 384]))
    gate = pick(["softmax", "sigmoid_group"])
    if gate == "sigmoid_group":
        n_group, per = int(pick([2, 4, 8])), int(pick([4, 8]))
        n_experts = n_group * per
        topk_group = int(g.integers(1, n_group + 1))
        top_k = int(g.integers(2, min(8, topk_group * per) + 1))
    else:
        n_group, topk_group = 1, 1
        n_experts = int(pick([8, 16, 24, 40, 64]))
        top_k = int(g.integers(2, min(8, n_experts) + 1))
    n_shared = int(pick([0, 0, 1, 2]))
    n_local = int(g.integers(max(1, n_experts // 2), n_experts + 1))
    spare = int(pick([0, 3]))
    n_slots = n_local + n_shared + spare
    tokens = int(pick([700, 1100, 1800, 2600, 3300]))
    b = int(g.integers(0, tokens // 2))
    e = int(g.integers(tokens // 2, tokens + 1))
    wl = MoEWorkload(name=f"big{i}", tokens=tokens, hidden=hidden, inter=inter, n_experts=n_experts, top_k=top_k,
                     n_slots=n_slots, n_local=n_local, act_dtype="bf16", router_dtype=pick(["f32", "bf16"]),
                     gate=gate, n_group=n_group, topk_group=topk_group, renormalize=bool(g.integers(2)),
                     routed_scale=float(pick([1.0, 2.5])), n_shared=n_shared, shared_range=(b, e) if n_shared else (0, 0),
                     zipf_s=float(pick([0.0, 1.2])), seed=6000 + i)
    local = np.sort(g.choice(n_experts, size=n_local, replace=False))
    slots = g.permutation(n_local + spare)[:n_local]
    emap = np.full(n_experts, -1, np.int32)
    emap[local] = slots
    return wl, emap, local


@pytest.mark.parametrize("i", range(24))
def test_random_shape(i):
    _check(*_random_case(i))


@pytest.mark.parametrize("i", range(10))
def test_random_large_shape(i):
    _check(*_random_large_case(i))


def _check(wl, emap, local):
    from gpu_util import Case, check_routing, check_bookkeeping, check_output
    from workloads import make_inputs
    # the generator draws weights for logical experts 0..n_local-1 (+ shared); hand expert local[j] the j-th set
    inp = make_inputs(wl)
    case = Case.__new__(Case)
    # build the slot pools by hand: Case.place assumes local experts are 0..n_local-1
    from oracle import LayerSpec
    from paper_2510_02613_amd.layer import MoELayer
    shared_slots = np.arange(wl.n_slots - wl.n_shared, wl.n_slots, dtype=np.int32)
    case.wl, case.inp, case.spec = wl, inp, LayerSpec.from_workload(wl)
    case.expert_map, case.shared_slots, case.select_bias = emap, shared_slots, None
    fill = np.float32(np.nan)
    def pool(experts):
        p = np.empty((wl.n_slots,) + experts.shape[1:], experts.dtype)
        p[...] = np.uint16(0x7fc0) if experts.dtype == np.uint16 else fill     # NaN in unused slots
        for j, e in enumerate(local):
            p[emap[e]] = experts[j]
        for s in range(wl.n_shared):
            p[shared_slots[s]] = experts[wl.n_local + s]
        return p
    case.w13_pool, case.w2_pool = pool(inp["w13_experts"]), pool(inp["w2_experts"])
    case.layer = MoELayer(hidden=wl.hidden, inter=wl.inter, n_experts=wl.n_experts, top_k=wl.top_k, n_slots=wl.n_slots,
                          max_tokens=wl.tokens, act_dtype=wl.act_dtype, router_dtype=wl.router_dtype, gate=wl.gate,
                          n_group=wl.n_group, topk_group=wl.topk_group, renormalize=wl.renormalize,
                          routed_scale=wl.routed_scale, n_shared=wl.n_shared, router_w=inp["router_w"],
                          logit_bias=inp["logit_bias"])
    case.layer.load_pool(case.w13_pool, case.w2_pool)
    case.layer.set_expert_map(emap, shared_slots if wl.n_shared else None)
    case.x_dev = case.layer.upload(inp["x"])
    out = case.run()
    v = case.layer.view(wl.tokens)
    ids, _, _ = check_routing(case, v["topk_ids"], v["topk_w"])
    check_bookkeeping(case, v, wl.tokens, wl.shared_range)
    check_output(case, out, ids)
    # the same pass with the assignments ranked by the separate histogram kernels (the path of routed passes and
    # of very large batches) instead of inside the selection kernel: same bookkeeping, same bits
    from paper_2510_02613_amd.binding import MOE_FLAG_PERMUTE_UNFUSED
    out2 = case.run(flags=MOE_FLAG_PERMUTE_UNFUSED)
    v2 = case.layer.view(wl.tokens)
    check_bookkeeping(case, v2, wl.tokens, wl.shared_range, MOE_FLAG_PERMUTE_UNFUSED)
    for key in ("topk_ids", "counts", "offsets", "perm", "inv"):
        np.testing.assert_array_equal(v[key], v2[key])
    np.testing.assert_array_equal(out, out2)
