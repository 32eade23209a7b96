"""Pins for the CPU oracle: things the mathematics fixes independently of it.

Every expected value here comes from a library routine (numpy / scipy / torch in
fp64), a closed form, a hand-worked example under tests/golden/, or a structural
invariant -- never from the oracle itself and never from the GPU path.
"""
import itertools
import os

import numpy as np
import pytest
import scipy.special
import torch

import oracle
from oracle import LayerSpec
from workloads import (f32_to_bf16_bits, bf16_bits_to_f32, get_workload, make_inputs,
                       build_slot_pool, block_expert_map)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rnd(seed):
    return np.random.Generator(np.random.PCG64(seed))


def small_layer(seed, T=13, H=24, I=10, E=6, k=2, S=None, **kw):
    """Random small layer with H, I, 2I all different (catches transposed operands)."""
    S = E if S is None else S
    g = rnd(seed)
    x = g.standard_normal((T, H)).astype(np.float32)
    wr = (g.standard_normal((E, H)) * 0.3).astype(np.float32)
    w13 = (g.standard_normal((S, 2 * I, H)) * 0.2).astype(np.float32)
    w2 = (g.standard_normal((S, H, I)) * 0.2).astype(np.float32)
    spec = LayerSpec(T=T, H=H, I=I, E=E, k=k, S=S, **kw)
    return spec, x, wr, w13, w2


def lib_ffn(x, w13, w2):
    """SwiGLU FFN from library ops in fp64: silu(x Wg^T) * (x Wu^T) W2^T."""
    I = w13.shape[0] // 2
    xt = torch.from_numpy(x.astype(np.float64))
    wg = torch.from_numpy(w13[:I].astype(np.float64))
    wu = torch.from_numpy(w13[I:].astype(np.float64))
    wd = torch.from_numpy(w2.astype(np.float64))
    h = torch.nn.functional.silu(xt @ wg.T) * (xt @ wu.T)
    return (h @ wd.T).numpy()


# ---------------------------------------------------------------- gating ----

def test_softmax_scores_and_order_match_library():
    spec, x, wr, *_ = small_layer(1, T=50, E=16, k=4)
    ids, w, flags, c = oracle.route(spec, x, wr, want_scores=True)
    logits = x.astype(np.float64) @ wr.astype(np.float64).T
    s = scipy.special.softmax(logits, axis=1)
    np.testing.assert_allclose(c, s.astype(np.float32), rtol=0, atol=1e-7)
    order = np.argsort(-s.astype(np.float32), axis=1, kind="stable")[:, :spec.k]
    ok = flags == 0
    assert ok.sum() > 40
    np.testing.assert_array_equal(ids[ok], order[ok])
    # distinct ids, weights sum to 1
    assert all(len(set(r)) == spec.k for r in ids)
    np.testing.assert_allclose(w.sum(1), 1.0, rtol=0, atol=1e-12)
    # closed form: softmax -> top-k -> renormalise == softmax over the k selected logits
    sel = np.take_along_axis(logits, ids.astype(np.int64), axis=1)
    np.testing.assert_allclose(w, scipy.special.softmax(sel, axis=1), rtol=0, atol=1e-13)


def test_k_equals_E_gives_full_softmax():
    spec, x, wr, *_ = small_layer(2, E=5, k=5)
    ids, w, _ = oracle.route(spec, x, wr)
    s = scipy.special.softmax(x.astype(np.float64) @ wr.astype(np.float64).T, axis=1)
    full = np.zeros_like(s)
    np.put_along_axis(full, ids.astype(np.int64), w, axis=1)
    np.testing.assert_allclose(full, s, rtol=0, atol=1e-14)


def test_no_renormalise_and_scale():
    spec, x, wr, *_ = small_layer(3, E=8, k=3, renormalize=False, routed_scale=1.75)
    ids, w, _ = oracle.route(spec, x, wr)
    s = scipy.special.softmax(x.astype(np.float64) @ wr.astype(np.float64).T, axis=1)
    np.testing.assert_allclose(w, 1.75 * np.take_along_axis(s, ids.astype(np.int64), 1),
                               rtol=0, atol=1e-14)


def test_logit_bias_is_added_before_softmax():
    spec, x, wr, *_ = small_layer(4, E=8, k=2)
    bias = rnd(40).standard_normal(8).astype(np.float32)
    ids, w, flags, c = oracle.route(spec, x, wr, logit_bias=bias, want_scores=True)
    s = scipy.special.softmax(x.astype(np.float64) @ wr.astype(np.float64).T
                              + bias.astype(np.float64), axis=1)
    np.testing.assert_allclose(c, s.astype(np.float32), rtol=0, atol=1e-7)
    np.testing.assert_allclose(w.sum(1), 1.0, atol=1e-12)


def test_select_bias_moves_selection_not_weights():
    spec, x, wr, *_ = small_layer(5, E=8, k=2, renormalize=False)
    sb = np.zeros(8, np.float32)
    sb[6] = 10.0  # expert 6 always wins selection
    ids, w, _ = oracle.route(spec, x, wr, select_bias=sb)
    assert (ids[:, 0] == 6).all()
    s = scipy.special.softmax(x.astype(np.float64) @ wr.astype(np.float64).T, axis=1)
    np.testing.assert_allclose(w[:, 0], s[:, 6], rtol=0, atol=1e-14)  # un-biased score


def test_sigmoid_gate_single_group_is_plain_sigmoid_topk():
    spec, x, wr, *_ = small_layer(6, T=40, E=12, k=3, gate="sigmoid_group", routed_scale=2.5)
    ids, w, flags, c = oracle.route(spec, x, wr, want_scores=True)
    s = scipy.special.expit(x.astype(np.float64) @ wr.astype(np.float64).T)
    np.testing.assert_allclose(c, s.astype(np.float32), rtol=0, atol=1e-7)
    order = np.argsort(-s.astype(np.float32), axis=1, kind="stable")[:, :3]
    ok = flags == 0
    np.testing.assert_array_equal(ids[ok], order[ok])
    sel = np.take_along_axis(s, ids.astype(np.int64), 1)
    np.testing.assert_allclose(w, 2.5 * sel / sel.sum(1, keepdims=True), rtol=0, atol=1e-13)
    np.testing.assert_allclose(w.sum(1), 2.5, atol=1e-12)


def _read_golden(name):
    d = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            d[key] = [float(v) for v in vals]
    return d


@pytest.mark.parametrize("k", [3, 2])
def test_grouped_gate_hand_worked_example(k):
    g = _read_golden("grouped_gate_example.txt")
    p = np.array(g["scores"], dtype=np.float64)
    E = p.size
    logits = np.log(p / (1 - p))
    # identity router so that the logits are exactly the input row (bf16/fp32 exactness
    # does not matter: the expected values only need 1e-6)
    x = logits[None, :].astype(np.float32)
    wr = np.eye(E, dtype=np.float32)
    spec = LayerSpec(T=1, H=E, I=1, E=E, k=k, S=E, gate="sigmoid_group",
                     n_group=int(g["n_group"][0]), topk_group=int(g["topk_group"][0]),
                     routed_scale=g["scale"][0])
    ids, w, flags = oracle.route(spec, x, wr)
    assert ids[0].tolist() == [int(v) for v in g[f"k{k}_ids"]]
    np.testing.assert_allclose(w[0], g[f"k{k}_weights"], rtol=0, atol=1e-6)
    assert (flags[0] & 1) == (1 if k == 2 else 0)


def test_grouped_gate_brute_force_over_group_subsets():
    """E=8, G=4, keep 2 groups: the kept pair of groups is the subset with the largest
    total top-2-sum score; the selected experts are the k best of its members."""
    T, E, G, KG, k = 200, 8, 4, 2, 3
    g = rnd(7)
    x = g.standard_normal((T, E)).astype(np.float32)
    wr = np.eye(E, dtype=np.float32)
    spec = LayerSpec(T=T, H=E, I=1, E=E, k=k, S=E, gate="sigmoid_group", n_group=G, topk_group=KG)
    ids, w, flags = oracle.route(spec, x, wr)
    s = scipy.special.expit(x.astype(np.float64)).astype(np.float32)
    per = E // G
    checked = 0
    for t in range(T):
        if flags[t]:
            continue
        gs = [np.sort(s[t, q * per:(q + 1) * per])[-2:].sum(dtype=np.float32) for q in range(G)]
        best = max(itertools.combinations(range(G), KG), key=lambda c: sum(float(gs[q]) for q in c))
        members = [e for q in best for e in range(q * per, (q + 1) * per)]
        want = sorted(members, key=lambda e: (-s[t, e], e))[:k]
        assert ids[t].tolist() == want
        assert len({e // per for e in ids[t]}) <= KG
        checked += 1
    assert checked > 150


def test_groups_of_one_expert_reduce_to_plain_topk():
    """n_group = E: a group's score is its only expert's score, so keeping the topk_group >= k best
    groups and then the k best experts is plain sigmoid top-k (library sort), and with topk_group = k
    the kept groups ARE the selection."""
    T, E = 120, 12
    g = rnd(41)
    x = g.standard_normal((T, E)).astype(np.float32)
    wr = np.eye(E, dtype=np.float32)
    s = scipy.special.expit(x.astype(np.float64)).astype(np.float32)
    for k, kg in ((3, 5), (4, 4), (1, 12)):
        spec = LayerSpec(T=T, H=E, I=1, E=E, k=k, S=E, gate="sigmoid_group", n_group=E, topk_group=kg)
        ids, w, flags, c = oracle.route(spec, x, wr, want_scores=True)
        np.testing.assert_array_equal(c, s)
        want = np.argsort(-s, axis=1, kind="stable")[:, :k]
        ok = flags == 0
        assert ok.sum() > 100
        np.testing.assert_array_equal(ids[ok], want[ok])
        np.testing.assert_allclose(w.sum(1), 1.0, atol=1e-12)
        # group flag (bit 1): the kg-th and (kg+1)-th SINGLE scores within 1e-5
        srt = -np.sort(-s, axis=1)
        if kg < E:
            np.testing.assert_array_equal((flags >> 1) & 1, (srt[:, kg - 1] - srt[:, kg] < 1e-5).astype(np.uint8))


def test_tie_break_lower_index_and_flag():
    # experts 1 and 3 have identical router rows -> identical scores for every token
    spec, x, wr, *_ = small_layer(8, T=30, E=4, k=1)
    wr[3] = wr[1]
    wr[0] = -5 * np.abs(wr[0])
    wr[2] = wr[1] * 0.5
    ids, w, flags, c = oracle.route(spec, x, wr, want_scores=True)
    for t in range(30):
        if c[t, 1] >= c[t].max():
            assert ids[t, 0] == 1 and (flags[t] & 1)
    assert ((flags & 1) == 1).sum() >= 5
    # well separated scores are not flagged
    spec2, x2, wr2, *_ = small_layer(9, T=30, E=4, k=1)
    wr2 *= 10
    ids2, w2, flags2, c2 = oracle.route(spec2, x2, wr2, want_scores=True)
    top2 = np.sort(c2, axis=1)[:, -2:]
    np.testing.assert_array_equal(flags2 & 1, (top2[:, 1] - top2[:, 0] < 1e-5).astype(np.uint8))


def test_tie_flag_threshold_is_1e_minus_5_on_fp32_scores():
    # two experts, softmax: score gap = tanh(d/2) ~ d/2 for logit gap d
    wr = np.array([[1.0], [0.0]], np.float32)
    spec = LayerSpec(T=2, H=1, I=1, E=2, k=1, S=2)
    x = np.array([[6e-6], [6e-5]], np.float32)  # gaps 3e-6 (flag) and 3e-5 (no flag)
    ids, w, flags = oracle.route(spec, x, wr)
    assert ids[:, 0].tolist() == [0, 0]
    assert (flags & 1).tolist() == [1, 0]
    # group flag (bit 1): 4 experts in 2 groups of 2, keep 1 group; group scores nearly equal
    p = np.array([[0.6, 0.3, 0.5, 0.400003], [0.6, 0.3, 0.5, 0.4001]])
    xg = np.log(p / (1 - p)).astype(np.float32)
    specg = LayerSpec(T=2, H=4, I=1, E=4, k=1, S=4, gate="sigmoid_group", n_group=2, topk_group=1)
    ids, w, flags = oracle.route(specg, xg, np.eye(4, dtype=np.float32))
    assert ids[:, 0].tolist() == [2, 2]          # group 1 wins (0.900003 / 0.9001 > 0.9)
    assert ((flags >> 1) & 1).tolist() == [1, 0]


# ------------------------------------------------------------- expert FFN ---

def test_single_expert_layer_is_one_swiglu_ffn():
    spec, x, wr, w13, w2 = small_layer(10, E=1, k=1)
    out = oracle.forward(spec, x, wr, w13, w2, np.zeros(1, np.int32))
    np.testing.assert_allclose(out, lib_ffn(x, w13[0], w2[0]), rtol=1e-12, atol=1e-13)


def test_dense_mixture_when_k_equals_E():
    spec, x, wr, w13, w2 = small_layer(11, E=4, k=4)
    out = oracle.forward(spec, x, wr, w13, w2, np.arange(4, dtype=np.int32))
    s = scipy.special.softmax(x.astype(np.float64) @ wr.astype(np.float64).T, axis=1)
    want = sum(s[:, e:e + 1] * lib_ffn(x, w13[e], w2[e]) for e in range(4))
    np.testing.assert_allclose(out, want, rtol=1e-11, atol=1e-13)


def test_topk_layer_against_library_per_expert():
    """General case from library pieces: ids/weights checked above, so combine them here."""
    spec, x, wr, w13, w2 = small_layer(12, T=21, E=6, k=2, S=9)
    emap = np.array([4, -1, 0, 8, -1, 2], np.int32)
    out = oracle.forward(spec, x, wr, w13, w2, emap)
    ids, w, _ = oracle.route(spec, x, wr)
    ffn = {s: lib_ffn(x, w13[s], w2[s]) for s in set(emap.tolist()) - {-1}}
    want = np.zeros_like(out)
    for t in range(spec.T):
        for j in range(spec.k):
            s = emap[ids[t, j]]
            if s >= 0:
                want[t] += w[t, j] * ffn[s][t]
    np.testing.assert_allclose(out, want, rtol=1e-11, atol=1e-13)


def test_shared_expert_weight_one_on_its_token_range_only():
    spec, x, wr, w13, w2 = small_layer(13, T=12, E=4, k=2, S=5, n_shared=1, routed_scale=2.5,
                                       gate="sigmoid_group")
    emap = np.arange(4, dtype=np.int32)
    base = oracle.forward(LayerSpec(**{**spec.__dict__, "n_shared": 0}), x, wr, w13, w2, emap)
    out = oracle.forward(spec, x, wr, w13, w2, emap, shared_slots=[4], shared_range=(3, 9))
    sh = lib_ffn(x, w13[4], w2[4])
    want = base.copy()
    want[3:9] += sh[3:9]  # weight 1.0, not multiplied by routed_scale
    np.testing.assert_allclose(out, want, rtol=1e-11, atol=1e-13)


def test_brute_force_scalar_loop_on_tiny_f32_workload():
    """An independent per-token scalar loop (python floats) on a cut of the tiny workload."""
    wl = get_workload("tiny_f32").with_tokens(6)
    inp = make_inputs(wl)
    x, wr, w13, w2 = inp["x"], inp["router_w"], inp["w13_experts"], inp["w2_experts"]
    spec = LayerSpec.from_workload(wl)
    emap = np.arange(wl.n_experts, dtype=np.int32)
    out = oracle.forward(spec, x, wr, w13, w2, emap)
    import math
    H, I, E, k = wl.hidden, wl.inter, wl.n_experts, wl.top_k
    for t in range(wl.tokens):
        lg = [math.fsum(float(x[t, h]) * float(wr[e, h]) for h in range(H)) for e in range(E)]
        m = max(lg)
        ex = [math.exp(v - m) for v in lg]
        z = math.fsum(ex)
        sc = [v / z for v in ex]
        top = sorted(range(E), key=lambda e: (-np.float32(sc[e]), e))[:k]
        den = math.fsum(sc[e] for e in top)
        row = [0.0] * H
        for e in top:
            a = []
            for i in range(I):
                gg = math.fsum(float(w13[e, i, h]) * float(x[t, h]) for h in range(H))
                uu = math.fsum(float(w13[e, I + i, h]) * float(x[t, h]) for h in range(H))
                a.append(gg / (1.0 + math.exp(-gg)) * uu)
            for h in range(H):
                row[h] += sc[e] / den * math.fsum(float(w2[e, h, i]) * a[i] for i in range(I))
        np.testing.assert_allclose(out[t], row, rtol=1e-10, atol=1e-15)


# ------------------------------------------------ permute / combine / map ---

def test_identity_experts_return_scaled_input():
    spec, x, wr, w13, w2 = small_layer(14, E=6, k=3)
    emap = np.arange(6, dtype=np.int32)
    out = oracle.forward(spec, x, wr, w13, w2, emap, identity_experts=True)
    np.testing.assert_allclose(out, x.astype(np.float64), rtol=0, atol=1e-12)  # sum w = 1
    # only part of the experts local: out = (sum of local weights) * x
    emap2 = np.array([0, -1, 1, -1, -1, 2], np.int32)
    out2 = oracle.forward(spec, x, wr, w13, w2, emap2, identity_experts=True)
    ids, w, _ = oracle.route(spec, x, wr)
    f = (w * (emap2[ids] >= 0)).sum(1, keepdims=True)
    np.testing.assert_allclose(out2, f * x, rtol=0, atol=1e-12)


def test_tokens_without_local_expert_get_zero_rows():
    spec, x, wr, w13, w2 = small_layer(15, T=40, E=8, k=2, S=2)
    emap = block_expert_map(8, 0, 2)
    out = oracle.forward(spec, x, wr, w13, w2, emap)
    ids, _, _ = oracle.route(spec, x, wr)
    none_local = (emap[ids] < 0).all(1)
    assert none_local.any() and not none_local.all()
    assert (out[none_local] == 0.0).all()
    assert (np.abs(out[~none_local]).max(1) > 0).all()


def test_slot_permutation_leaves_output_unchanged():
    spec, x, wr, w13e, w2e = small_layer(16, T=17, E=6, k=2, S=6)
    S = 9
    spec = LayerSpec(**{**spec.__dict__, "S": S})
    m1 = np.arange(6, dtype=np.int32)
    m2 = np.array([7, 2, 8, 0, 5, 3], np.int32)
    outs = []
    for m in (m1, m2):
        p13 = build_slot_pool(w13e, m, S, 6)
        p2 = build_slot_pool(w2e, m, S, 6)
        outs.append(oracle.forward(spec, x, wr, p13, p2, m))
    np.testing.assert_array_equal(outs[0], outs[1])  # same arithmetic, same order: bit equal


def test_expert_parallel_ranks_sum_to_the_full_layer():
    """Sum over ranks of the per-rank partial outputs (block placement, shared expert on the
    rank's own share of the tokens) equals the EP=1 layer."""
    T, E, R = 16, 8, 4
    spec, x, wr, w13e, w2e = small_layer(17, T=T, E=E, k=3, S=E + 1, gate="sigmoid_group",
                                         n_group=4, topk_group=2, routed_scale=2.5, n_shared=1)
    full = oracle.forward(spec, x, wr, w13e, w2e, np.arange(E, dtype=np.int32),
                          shared_slots=[E], shared_range=(0, T))
    per = E // R
    acc = np.zeros_like(full)
    rspec = LayerSpec(**{**spec.__dict__, "S": per + 1})
    for r in range(R):
        m = block_expert_map(E, r * per, per)
        p13 = np.concatenate([w13e[r * per:(r + 1) * per], w13e[E:E + 1]])
        p2 = np.concatenate([w2e[r * per:(r + 1) * per], w2e[E:E + 1]])
        acc += oracle.forward(rspec, x, wr, p13, p2, m, shared_slots=[per],
                              shared_range=(r * T // R, (r + 1) * T // R))
    np.testing.assert_allclose(acc, full, rtol=1e-12, atol=1e-14)


def test_rows_are_independent_and_token_subsets_work():
    spec, x, wr, w13, w2 = small_layer(18, T=20, E=6, k=2)
    emap = np.arange(6, dtype=np.int32)
    full = oracle.forward(spec, x, wr, w13, w2, emap)
    tok = np.array([17, 3, 3, 0], np.int32)
    np.testing.assert_array_equal(oracle.forward(spec, x, wr, w13, w2, emap, tokens=tok), full[tok])
    # changing other tokens does not change row 5
    x2 = x.copy()
    x2[np.arange(20) != 5] += 1.0
    np.testing.assert_array_equal(oracle.forward(spec, x2, wr, w13, w2, emap, tokens=[5]), full[5:6])


def test_forced_ids_reproduce_own_routing_and_follow_other_routing():
    spec, x, wr, w13, w2 = small_layer(19, T=10, E=6, k=2)
    emap = np.arange(6, dtype=np.int32)
    ids, w, _ = oracle.route(spec, x, wr)
    full = oracle.forward(spec, x, wr, w13, w2, emap)
    np.testing.assert_array_equal(oracle.forward(spec, x, wr, w13, w2, emap, forced_ids=ids), full)
    forced = np.tile(np.array([[5, 1]], np.int32), (10, 1))
    out = oracle.forward(spec, x, wr, w13, w2, emap, forced_ids=forced)
    s = scipy.special.softmax(x.astype(np.float64) @ wr.astype(np.float64).T, axis=1)
    den = s[:, 5] + s[:, 1]
    want = (s[:, 5] / den)[:, None] * lib_ffn(x, w13[5], w2[5]) + \
           (s[:, 1] / den)[:, None] * lib_ffn(x, w13[1], w2[1])
    np.testing.assert_allclose(out, want, rtol=1e-11, atol=1e-13)


def test_bf16_storage_is_widened_exactly():
    spec, x, wr, w13, w2 = small_layer(20, T=9, E=4, k=2)
    xb, w13b, w2b, wrb = (f32_to_bf16_bits(a) for a in (x, w13, w2, wr))
    emap = np.arange(4, dtype=np.int32)
    a = oracle.forward(spec, xb, wrb, w13b, w2b, emap)
    b = oracle.forward(spec, bf16_bits_to_f32(xb), bf16_bits_to_f32(wrb),
                       bf16_bits_to_f32(w13b), bf16_bits_to_f32(w2b), emap)
    np.testing.assert_array_equal(a, b)
    # mixed: bf16 activations/weights with an fp32 router
    c = oracle.forward(spec, xb, bf16_bits_to_f32(wrb), w13b, w2b, emap)
    np.testing.assert_array_equal(a, c)


def test_bf16_rounding_helper_matches_torch():
    v = rnd(21).standard_normal(4096).astype(np.float32) * 3
    v[:4] = [0.0, -0.0, 1.0, 2.0 ** -130]
    ours = f32_to_bf16_bits(v)
    theirs = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(ours, theirs)
    back = torch.from_numpy(theirs.view(np.int16)).view(torch.bfloat16).float().numpy()
    np.testing.assert_array_equal(bf16_bits_to_f32(ours), back)


# ------------------------------------------------- routing given (steps 5-7) ----

def test_routed_entry_against_library_ffn_with_arbitrary_ids_and_weights():
    """Given ids and weights, a row is sum_j w_j * FFN_{map[id_j]}(x_t) from library ops;
    remote experts (-1 in the map) and padding ids (outside [0,E)) add nothing; a repeated id counts twice."""
    spec, x, wr, w13, w2 = small_layer(41, T=9, E=6, k=3, S=8)
    g = rnd(42)
    emap = np.array([5, -1, 0, 7, 2, -1], dtype=np.int32)          # experts 1 and 5 remote, slots scattered
    ids = g.integers(0, spec.E, size=(spec.T, spec.k)).astype(np.int32)
    ids[0] = [3, 3, 1]          # repeated id, remote id
    ids[1] = [-1, 6, 2]         # two padding ids
    wts = g.uniform(-1.0, 2.0, size=(spec.T, spec.k)).astype(np.float32)   # not normalised, may be negative
    got = oracle.forward_routed(spec, x, w13, w2, emap, ids, wts)
    want = np.zeros((spec.T, spec.H))
    for t in range(spec.T):
        for j in range(spec.k):
            e = ids[t, j]
            if 0 <= e < spec.E and emap[e] >= 0:
                want[t] += float(wts[t, j]) * lib_ffn(x[t:t + 1], w13[emap[e]], w2[emap[e]])[0]
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_routed_entry_identity_experts_and_shared_range():
    """Identity experts: row = (sum of the weights of local, existing ids + 1 per shared expert in range) * x."""
    spec, x, wr, w13, w2 = small_layer(43, T=7, E=4, k=2, S=6, n_shared=1)
    emap = np.array([0, 1, -1, 3], dtype=np.int32)
    ids = np.array([[0, 1], [2, 3], [3, 3], [9, 0], [1, 2], [2, 2], [0, 3]], dtype=np.int32)
    wts = rnd(44).uniform(0.1, 1.0, size=ids.shape).astype(np.float32)
    got = oracle.forward_routed(spec, x, w13, w2, emap, ids, wts, shared_slots=[5], shared_range=(2, 5),
                                identity_experts=True)
    for t in range(spec.T):
        coef = sum(float(wts[t, j]) for j in range(spec.k) if 0 <= ids[t, j] < spec.E and emap[ids[t, j]] >= 0)
        coef += 1.0 if 2 <= t < 5 else 0.0
        np.testing.assert_allclose(got[t], coef * x[t].astype(np.float64), rtol=1e-13, atol=1e-13)


def test_routed_entry_with_own_routing_equals_the_gated_layer():
    """Feeding the gate's own ids and (fp32-exact) weights back reproduces the gated layer."""
    spec, x, wr, w13, w2 = small_layer(45, T=11, E=8, k=3, S=8)
    emap = np.arange(8, dtype=np.int32)
    ids, w, _ = oracle.route(spec, x, wr)
    w32 = w.astype(np.float32)
    full = oracle.forward(spec, x, wr, w13, w2, emap)
    routed = oracle.forward_routed(spec, x, w13, w2, emap, ids, w32)
    # only difference: the weights were rounded to fp32 on the way
    np.testing.assert_allclose(routed, full, rtol=0, atol=2e-7 * np.abs(full).max())
    sub = np.array([7, 2, 2, 10], dtype=np.int32)
    np.testing.assert_array_equal(oracle.forward_routed(spec, x, w13, w2, emap, ids, w32, tokens=sub), routed[sub])


# --------------------------------------------- replicated placement (step 5) ----

def test_replicated_placement_against_library_ffn_with_distinct_copies():
    """Copies that hold DIFFERENT weights expose which copy a token uses: row t is
    sum_j w_j * FFN_{replicas[e_j][t mod R]}(x_t) from library ops, experts with no copy add nothing."""
    spec, x, wr, w13, w2 = small_layer(51, T=17, E=5, k=2, S=9)
    replicas = [[4], [0, 7, 2], [], [8, 1], [3]]
    g = rnd(52)
    forced = np.stack([g.choice(spec.E, size=spec.k, replace=False) for _ in range(spec.T)]).astype(np.int32)
    got = oracle.forward_replicated(spec, x, wr, w13, w2, replicas, forced_ids=forced)
    # weights from the gate definition, library softmax in fp64
    s = scipy.special.softmax(x.astype(np.float64) @ wr.astype(np.float64).T, axis=1)
    want = np.zeros((spec.T, spec.H))
    used = set()
    for t in range(spec.T):
        wsum = sum(s[t, e] for e in forced[t])
        for e in forced[t]:
            if replicas[e]:
                slot = replicas[e][t % len(replicas[e])]
                used.add(slot)
                want[t] += s[t, e] / wsum * lib_ffn(x[t:t + 1], w13[slot], w2[slot])[0]
    assert used == {0, 1, 2, 3, 4, 7, 8}          # every copy is exercised
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-12)


def test_replicated_placement_with_equal_copies_is_the_unreplicated_layer():
    """Replication must not change the function: with identical weights in all copies of an expert the
    output equals that of the plain map, bit for bit, whatever the number of copies."""
    spec, x, wr, w13, w2 = small_layer(53, T=23, E=6, k=3, S=12, gate="sigmoid_group", n_group=2, topk_group=1,
                                       routed_scale=2.5, n_shared=1)
    emap = np.array([0, 1, -1, 3, 4, 5], dtype=np.int32)
    replicas = [[0, 6, 7], [1], [], [3, 8], [4, 9, 10, 11], [5]]
    for e, r in enumerate(replicas):
        for s_ in r[1:]:
            w13[s_] = w13[r[0]]
            w2[s_] = w2[r[0]]
    plain = oracle.forward(spec, x, wr, w13, w2, emap, shared_slots=[2], shared_range=(4, 20))
    rep = oracle.forward_replicated(spec, x, wr, w13, w2, replicas, shared_slots=[2], shared_range=(4, 20))
    np.testing.assert_array_equal(rep, plain)
    # and a placement with at most one copy everywhere IS the plain map
    single = oracle.forward_replicated(spec, x, wr, w13, w2, [[s_] if s_ >= 0 else [] for s_ in emap],
                                       shared_slots=[2], shared_range=(4, 20))
    np.testing.assert_array_equal(single, plain)


def test_replicated_placement_identity_experts_and_token_subset():
    spec, x, wr, w13, w2 = small_layer(54, T=10, E=4, k=2, S=6, renormalize=False)
    replicas = [[0, 1], [], [2, 3, 4], [5]]
    ids, w, _ = oracle.route(spec, x, wr)
    got = oracle.forward_replicated(spec, x, wr, w13, w2, replicas, identity_experts=True)
    for t in range(spec.T):
        coef = sum(w[t, j] for j in range(spec.k) if replicas[ids[t, j]])
        np.testing.assert_allclose(got[t], coef * x[t].astype(np.float64), rtol=1e-13, atol=1e-13)
    full = oracle.forward_replicated(spec, x, wr, w13, w2, replicas)
    sub = np.array([9, 0, 4, 4], dtype=np.int32)
    np.testing.assert_array_equal(oracle.forward_replicated(spec, x, wr, w13, w2, replicas, tokens=sub), full[sub])
