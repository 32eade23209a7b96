"""GPU parity of the pass that takes its routing from the caller (moe_forward_routed) against the
oracle's routed entry on the same seeded inputs, ids and weights."""
import numpy as np
import pytest

import oracle
from workloads import MoEWorkload, get_workload

pytestmark = pytest.mark.gpu

SMALL = dict(hidden=256, inter=136, n_experts=16, top_k=4, n_slots=16, n_local=16,
             act_dtype="bf16", router_dtype="f32", gate="softmax", seed=21)


def _routing(wl, seed, pad_frac=0.1):
    """Seeded ids with padding entries, out-of-range ids and repeats, and un-normalised signed weights."""
    g = np.random.Generator(np.random.PCG64(seed))
    ids = g.integers(0, wl.n_experts, size=(wl.tokens, wl.top_k)).astype(np.int32)
    pad = g.random(ids.shape) < pad_frac
    ids[pad] = np.where(g.random(int(pad.sum())) < 0.5, -1, wl.n_experts + 3)
    if wl.tokens > 2:
        ids[1, :] = ids[1, 0]                      # one expert k times
        ids[2, :] = -1                             # a token with no assignment at all
    wts = g.uniform(-0.5, 1.5, size=ids.shape).astype(np.float32)
    return ids, wts


def _run_routed(case, ids, wts, T=None, shared_range=None, flags=0):
    import torch
    from gpu_util import tensor_to_host
    T = case.wl.tokens if T is None else T
    sr = case.wl.shared_range if shared_range is None else shared_range
    dev = case.x_dev.device
    d_ids = torch.from_numpy(np.ascontiguousarray(ids[:T])).to(dev)
    d_w = torch.from_numpy(np.ascontiguousarray(wts[:T])).to(dev)
    out = case.layer.forward_routed(case.x_dev[:T], d_ids, d_w, shared_range=sr, flags=flags)
    torch.cuda.synchronize()
    return tensor_to_host(out)


def _check(case, ids, wts, sample=None, identity=False, flags=0):
    from gpu_util import to_f64, rel_err, TOL
    wl = case.wl
    got_bits = _run_routed(case, ids, wts, flags=flags)
    tokens = None
    if sample is not None and sample < wl.tokens:
        g = np.random.Generator(np.random.PCG64(777 + wl.seed))
        tokens = np.sort(g.choice(wl.tokens, size=sample, replace=False)).astype(np.int32)
    want = oracle.forward_routed(case.spec, case.inp["x"], case.w13_pool, case.w2_pool, case.expert_map, ids, wts,
                                 shared_slots=case.shared_slots, shared_range=wl.shared_range, tokens=tokens,
                                 identity_experts=identity)
    got = to_f64(got_bits if tokens is None else got_bits[tokens])
    assert np.isfinite(got).all()
    err = rel_err(got, want)
    assert err <= TOL[wl.act_dtype], f"max relative error {err:.3e}"
    zero = np.abs(want).max(1) == 0
    assert (got[zero] == 0).all()
    # slot histogram of the pass against its definition
    v = case.layer.view(wl.tokens)
    valid = (ids >= 0) & (ids < wl.n_experts)
    slot = np.where(valid, case.expert_map[np.clip(ids, 0, wl.n_experts - 1)], -1)
    counts = np.bincount(slot[slot >= 0], minlength=wl.n_slots)
    for i in range(wl.n_shared):
        counts[case.shared_slots[i]] += wl.shared_range[1] - wl.shared_range[0]
    np.testing.assert_array_equal(v["counts"], counts)
    return got_bits


@pytest.mark.parametrize("tokens", [5, 300, 2500])
def test_routed_small_bf16_arbitrary_ids_and_weights(tokens):
    """decode-sized, mid-sized and large-tile dispatch; padding ids, repeated ids, signed weights"""
    from gpu_util import Case
    wl = MoEWorkload(name="routed_small", tokens=tokens, **SMALL)
    emap = np.arange(16, dtype=np.int32)
    emap[[3, 9]] = -1                             # two experts live on another rank
    case = Case(wl, expert_map=emap)
    ids, wts = _routing(wl, 100 + tokens)
    _check(case, ids, wts)


def test_routed_f32_layer_with_shared_expert():
    from gpu_util import Case
    wl = MoEWorkload(name="routed_f32", tokens=77, hidden=136, inter=72, n_experts=8, top_k=3, n_slots=10, n_local=8,
                     act_dtype="f32", router_dtype="f32", gate="softmax", n_shared=1, shared_range=(10, 60), seed=22)
    case = Case(wl)
    ids, wts = _routing(wl, 5)
    _check(case, ids, wts)


def test_routed_identity_experts_closed_form():
    """out = (sum of the weights of existing local ids) * x"""
    from gpu_util import Case
    wl = MoEWorkload(name="routed_id", tokens=200, **SMALL)
    case = Case(wl)
    ids, wts = _routing(wl, 9)
    from paper_2510_02613_amd import binding as B
    _check(case, ids, wts, identity=True, flags=B.MOE_FLAG_IDENTITY_EXPERTS)


def test_routed_with_the_gates_own_routing_is_bit_identical_to_the_gated_pass():
    from gpu_util import Case
    wl = MoEWorkload(name="routed_self", tokens=700, **SMALL)
    case = Case(wl)
    gated = case.run()
    v = case.layer.view(wl.tokens)
    routed = _run_routed(case, v["topk_ids"], v["topk_w"])
    np.testing.assert_array_equal(routed, gated)


def test_routed_qwen3_shape_full_size_sampled():
    """Headline shapes: the oracle's own routing (weights rounded to fp32) fed to both sides."""
    from gpu_util import Case
    wl = get_workload("qwen3_30b_a3b")
    case = Case(wl)
    ids, w, _, _ = case.oracle_route()
    _check(case, ids, w.astype(np.float32), sample=96)


def test_routed_rejects_missing_routing():
    import torch
    from gpu_util import Case
    from paper_2510_02613_amd import binding as B
    wl = MoEWorkload(name="routed_err", tokens=8, **SMALL)
    case = Case(wl)
    out = torch.empty_like(case.x_dev)
    with pytest.raises(B.MoEError):
        B.moe_forward_routed(case.layer.handle, case.x_dev.data_ptr(), 8, 0, 0, out.data_ptr())
