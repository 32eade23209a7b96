"""Replicated placement on the GPU (moe_set_expert_replicas): an expert held in several slots, token t
using copy t mod R.  Copies are given DIFFERENT weights where the choice of copy is what is tested, and
equal weights where the claim is that replication does not change the layer."""
import numpy as np
import pytest

from workloads import MoEWorkload, make_inputs

pytestmark = pytest.mark.gpu


def _layer(wl, inp):
    from paper_2510_02613_amd.layer import MoELayer
    return MoELayer(hidden=wl.hidden, inter=wl.inter, n_experts=wl.n_experts, top_k=wl.top_k, n_slots=wl.n_slots,
                    max_tokens=wl.tokens, act_dtype=wl.act_dtype, router_dtype=wl.router_dtype, gate=wl.gate,
                    n_group=wl.n_group, topk_group=wl.topk_group, renormalize=wl.renormalize,
                    routed_scale=wl.routed_scale, n_shared=wl.n_shared, router_w=inp["router_w"],
                    logit_bias=inp["logit_bias"])


def _random_pool(g, shape, act):
    from workloads import f32_to_bf16_bits
    w = (g.standard_normal(shape) * 0.02).astype(np.float32)
    return f32_to_bf16_bits(w) if act == "bf16" else w


def _placement(g, n_experts, n_slots, n_shared, n_remote, max_copies):
    """Random placement: n_remote experts without a copy, the others 1..max_copies copies in scattered slots."""
    slots = list(g.permutation(n_slots - n_shared))
    remote = set(int(e) for e in g.choice(n_experts, size=n_remote, replace=False))
    want = [0 if e in remote else 1 for e in range(n_experts)]
    spare = len(slots) - sum(want)
    assert spare >= 0
    while spare > 0:
        e = int(g.integers(n_experts))
        if 0 < want[e] < max_copies:
            want[e] += 1
            spare -= 1
        elif all(w == 0 or w >= max_copies for w in want):
            break
    return [[int(slots.pop()) for _ in range(w)] for w in want]


def _slot_of(replicas, ids, T):
    t = np.arange(T)[:, None]
    R = np.array([len(r) for r in replicas])
    width = max(1, R.max())
    tab = np.full((len(replicas), width), -1, np.int64)
    for e, r in enumerate(replicas):
        tab[e, :len(r)] = r
    Rt = R[ids]
    return np.where(Rt > 0, tab[ids, t % np.maximum(Rt, 1)], -1)


CASES = [
    # name, act, T, H, I, E, k, S, shared, remote, max copies, gate
    ("generic_f32", "f32", 150, 64, 40, 8, 2, 16, 1, 1, 3, "softmax"),
    ("one_block_bf16", "bf16", 33, 128, 64, 16, 4, 30, 0, 3, 4, "softmax"),
    ("mfma_bf16", "bf16", 700, 256, 136, 24, 4, 40, 2, 4, 3, "sigmoid_group"),
    ("large_tiles_bf16", "bf16", 2600, 256, 128, 16, 6, 30, 1, 2, 5, "softmax"),
    ("many_copies_one_expert", "bf16", 900, 192, 64, 4, 2, 12, 0, 0, 9, "softmax"),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_distinct_copies_follow_the_choice_rule(case):
    """Every slot holds its own random weights, so the output is right only if each assignment went to
    copy t mod R of its expert; counts per slot are checked against the same rule."""
    import torch
    import oracle
    from oracle import LayerSpec
    from gpu_util import Case, check_routing, tensor_to_host, to_f64, rel_err, TOL
    name, act, T, H, I, E, k, S, n_shared, n_remote, max_copies, gate = case
    g = np.random.Generator(np.random.PCG64(sum(map(ord, name))))
    grouped = gate == "sigmoid_group"
    wl = MoEWorkload(name=name, tokens=T, hidden=H, inter=I, n_experts=E, top_k=k, n_slots=S, n_local=1,
                     act_dtype=act, router_dtype="f32", gate=gate, n_group=4 if grouped else 1,
                     topk_group=2 if grouped else 1, routed_scale=2.5 if grouped else 1.0, n_shared=n_shared,
                     shared_range=(T // 5, T - T // 7) if n_shared else (0, 0), seed=77)
    inp = make_inputs(wl)
    replicas = _placement(g, E, S, n_shared, n_remote, max_copies)
    shared_slots = np.arange(S - n_shared, S, dtype=np.int32)
    w13 = _random_pool(g, (S, 2 * I, H), act)
    w2 = _random_pool(g, (S, H, I), act)
    layer = _layer(wl, inp)
    layer.load_pool(w13, w2)
    layer.set_expert_replicas(replicas, shared_slots if n_shared else None)
    x_dev = layer.upload(inp["x"])
    out = layer.forward(x_dev, shared_range=wl.shared_range)
    torch.cuda.synchronize()
    out = tensor_to_host(out)
    v = layer.view(T)

    c = Case.__new__(Case)
    c.wl, c.inp, c.spec, c.select_bias = wl, inp, LayerSpec.from_workload(wl), None
    ids, _, _ = check_routing(c, v["topk_ids"], v["topk_w"])
    # bookkeeping under the rule: rows per slot, and every grouped row sits in the range of the slot it was sent to
    slot = np.full((T, k + n_shared), -1, np.int64)
    slot[:, :k] = _slot_of(replicas, ids, T)
    for i in range(n_shared):
        slot[wl.shared_range[0]:wl.shared_range[1], k + i] = shared_slots[i]
    counts = np.bincount(slot[slot >= 0], minlength=S)
    np.testing.assert_array_equal(v["counts"], counts)
    inv, offs = v["inv"], v["offsets"]
    np.testing.assert_array_equal(inv >= 0, slot >= 0)
    np.testing.assert_array_equal(np.searchsorted(offs, inv[inv >= 0], side="right") - 1, slot[inv >= 0])

    want = oracle.forward_replicated(c.spec, inp["x"], inp["router_w"], w13, w2, replicas,
                                     logit_bias=inp["logit_bias"], shared_slots=shared_slots[:n_shared],
                                     shared_range=wl.shared_range, forced_ids=ids)
    got = to_f64(out)
    assert np.isfinite(got).all()
    assert rel_err(got, want) <= TOL[act]
    layer.close()


def test_equal_copies_do_not_change_the_layer_and_switching_reallocates_nothing():
    """Zipf-skewed routing, the hottest experts copied into spare slots: the output is bit-identical to the
    plain placement's (a row's arithmetic does not depend on which group it sits in), matches the oracle,
    and going plain -> replicated -> plain touches neither the pools nor the workspace."""
    import torch
    from gpu_util import Case, check_routing, check_output
    wl = MoEWorkload(name="zipf_copies", tokens=3000, hidden=256, inter=128, n_experts=32, top_k=4, n_slots=44,
                     n_local=32, act_dtype="bf16", router_dtype="f32", gate="softmax", zipf_s=1.2, seed=91)
    case = Case(wl)                               # experts 0..31 in slots 0..31; 12 spare slots
    out_plain = case.run()
    v = case.layer.view(wl.tokens)
    ids, _, _ = check_routing(case, v["topk_ids"], v["topk_w"])
    check_output(case, out_plain, ids)
    load = np.bincount(ids.ravel(), minlength=wl.n_experts)
    hot = np.argsort(-load)[:4]
    replicas = [[e] for e in range(wl.n_experts)]
    spare = list(range(32, 44))
    for e in hot:                                  # 3 more copies of each of the 4 hottest experts
        for _ in range(3):
            s = spare.pop()
            replicas[e].append(s)
            case.layer.load_slot(s, case.w13_pool[e], case.w2_pool[e])
    ptrs = (case.layer.w13.data_ptr(), case.layer.w2.data_ptr(), case.layer.workspace.data_ptr())
    case.layer.set_expert_replicas(replicas)
    out_rep = case.run()
    vr = case.layer.view(wl.tokens)
    np.testing.assert_array_equal(vr["topk_ids"], v["topk_ids"])
    np.testing.assert_array_equal(out_rep, out_plain)
    # the hot experts' rows are now spread over their copies, evenly up to the spread of t mod 4
    for e in hot:
        per_copy = vr["counts"][replicas[e]]
        assert per_copy.sum() == load[e]
        assert per_copy.max() - per_copy.min() <= 4 * np.sqrt(load[e] / 4) + 4, per_copy
    assert vr["counts"][:32].max() < v["counts"][:32].max()          # the largest group shrank
    case.layer.set_expert_map(case.expert_map)
    np.testing.assert_array_equal(case.run(), out_plain)
    assert ptrs == (case.layer.w13.data_ptr(), case.layer.w2.data_ptr(), case.layer.workspace.data_ptr())
    torch.cuda.synchronize()


def test_replicated_placement_with_routing_given():
    """The pre-routed entry reads the same table: ids from the caller, copy by token index."""
    import torch
    import oracle
    from oracle import LayerSpec
    from gpu_util import tensor_to_host, to_f64, rel_err, TOL
    T, H, I, E, k, S = 500, 128, 64, 10, 3, 24
    wl = MoEWorkload(name="routed_copies", tokens=T, hidden=H, inter=I, n_experts=E, top_k=k, n_slots=S, n_local=1,
                     act_dtype="bf16", router_dtype="f32", gate="softmax", seed=5)
    inp = make_inputs(wl)
    g = np.random.Generator(np.random.PCG64(123))
    replicas = _placement(g, E, S, 0, 2, 4)
    w13, w2 = _random_pool(g, (S, 2 * I, H), "bf16"), _random_pool(g, (S, H, I), "bf16")
    ids = g.integers(-1, E + 1, size=(T, k)).astype(np.int32)       # includes padding ids on both sides
    wts = g.uniform(0.0, 1.0, size=(T, k)).astype(np.float32)
    layer = _layer(wl, inp)
    layer.load_pool(w13, w2)
    layer.set_expert_replicas(replicas)
    out = layer.forward_routed(layer.upload(inp["x"]), torch.from_numpy(ids).to(layer.device),
                               torch.from_numpy(wts).to(layer.device))
    torch.cuda.synchronize()
    # oracle: the routed entry with, per token, the plain map that the rule selects
    spec = LayerSpec.from_workload(wl)
    want = np.zeros((T, H))
    R = max(len(r) for r in replicas)
    for phase in range(int(np.lcm.reduce([max(1, len(r)) for r in replicas]))):
        emap = np.array([r[phase % len(r)] if r else -1 for r in replicas], np.int32)
        toks = np.arange(phase, T, int(np.lcm.reduce([max(1, len(r)) for r in replicas])), dtype=np.int32)
        if toks.size:
            want[toks] = oracle.forward_routed(spec, inp["x"], w13, w2, emap, ids, wts, tokens=toks)
    assert R >= 2
    assert rel_err(to_f64(tensor_to_host(out)), want) <= TOL["bf16"]
    layer.close()
