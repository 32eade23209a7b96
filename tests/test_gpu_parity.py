"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle on the same
seeded inputs.  Integer results (routing, bookkeeping) are bit exact up to flagged score
near-ties; outputs meet max-relative-error 1e-2 (bf16) / 1e-4 (fp32)."""

import numpy as np
import pytest

from workloads import MoEWorkload, get_workload, block_expert_map, relayout_maps

pytestmark = pytest.mark.gpu


def _case(wl, **kw):
    from gpu_util import Case
    return Case(wl, **kw)


def _tile_sample(v, rows_per_tile, extra_tokens, T, seed):
    """Tokens that cover EVERY M-tile of the pass: the first, the last and seeded random rows of each
    tile (a tile-position mistake cannot hide between samples), plus seeded tokens drawn from the whole batch
    (among them tokens with no local work, whose rows must be exactly zero)."""
    g = np.random.Generator(np.random.PCG64(seed))
    rows = []
    for _, r0, n, _ in v["tiles"]:
        pick = {int(r0), int(r0 + n - 1)}
        pick |= set(int(r) for r in r0 + g.choice(n, size=min(n, rows_per_tile), replace=False))
        rows.extend(sorted(pick))
    tok = set(int(t) for t in v["perm"][np.asarray(rows, np.int64)]) if rows else set()
    tok |= set(int(t) for t in g.choice(T, size=min(T, extra_tokens), replace=False))
    return np.array(sorted(tok), np.int32)


def _full_check(case, flags=0, sample=None, T=None, shared_range=None, report=None):
    """sample: None = every token is graded; an int = that many seeded tokens; ("tiles", r, x) = r rows of
    every M-tile plus x tokens of the whole batch."""
    from gpu_util import check_routing, check_bookkeeping, check_output
    wl = case.wl
    T = wl.tokens if T is None else T
    sr = wl.shared_range if shared_range is None else shared_range
    out = case.run(flags=flags, T=T, shared_range=sr)
    v = case.layer.view(T)
    if T == wl.tokens:
        grade_ids, n_flag, flips = check_routing(case, v["topk_ids"], v["topk_w"])
    else:
        grade_ids, n_flag, flips = None, 0, 0
    check_bookkeeping(case, v, T, sr, flags)
    tokens = None if T == wl.tokens else np.arange(T, dtype=np.int32)
    if isinstance(sample, tuple):
        tokens = _tile_sample(v, sample[1], sample[2], T, 1234 + wl.seed)
    elif sample is not None and sample < T:
        g = np.random.Generator(np.random.PCG64(1234 + wl.seed))
        tokens = np.sort(g.choice(T, size=sample, replace=False)).astype(np.int32)
    err = check_output(case, out, grade_ids, tokens=tokens, shared_range=sr, report=report)
    return out, v, err


SMALL = dict(hidden=256, inter=136, n_experts=16, top_k=4, n_slots=16, n_local=16,
             act_dtype="bf16", router_dtype="f32", gate="softmax", seed=11)


def test_tiny_f32_workload_all_tokens():
    case = _case(get_workload("tiny_f32"))
    _full_check(case)


@pytest.mark.parametrize("tokens", [1, 7, 300, 1000])
def test_small_bf16_softmax_ragged(tokens):
    wl = MoEWorkload(name="small", tokens=tokens, **SMALL)
    _full_check(_case(wl))


def test_small_f32_ragged_tiles():
    wl = MoEWorkload(name="small32", tokens=333, **{**SMALL, "act_dtype": "f32", "hidden": 136, "inter": 72})
    _full_check(_case(wl))


def test_small_grouped_sigmoid_with_shared_expert_and_partial_locality():
    wl = MoEWorkload(name="smallg", tokens=515, hidden=256, inter=136, n_experts=32, top_k=4,
                     n_slots=9, n_local=8, act_dtype="bf16", router_dtype="bf16",
                     gate="sigmoid_group", n_group=4, topk_group=2, routed_scale=2.5, n_shared=1,
                     shared_range=(100, 317), seed=12)
    case = _case(wl)
    out, v, _ = _full_check(case)
    # tokens with no local expert and outside the shared range are exact zero rows
    local = (case.expert_map[v["topk_ids"]] >= 0).any(1)
    outside = np.ones(wl.tokens, bool)
    outside[100:317] = False
    assert (outside & ~local).any()
    assert (out[outside & ~local] == 0).all()


def test_no_renormalise_scale_and_select_bias():
    wl = MoEWorkload(name="smallb", tokens=200, **{**SMALL, "renormalize": False, "routed_scale": 1.5})
    sb = np.zeros(16, np.float32)
    sb[3] = 0.5
    case = _case(wl, select_bias=sb)
    out, v, _ = _full_check(case)
    assert (v["topk_ids"] == 3).any(1).all()


def test_identity_experts_return_weighted_input():
    from gpu_util import check_output, check_routing, to_f64
    from paper_2510_02613_amd import MOE_FLAG_IDENTITY_EXPERTS
    wl = MoEWorkload(name="ident", tokens=300, **{**SMALL, "act_dtype": "f32"})
    case = _case(wl)
    out = case.run(flags=MOE_FLAG_IDENTITY_EXPERTS)
    v = case.layer.view(wl.tokens)
    ids, _, _ = check_routing(case, v["topk_ids"], v["topk_w"])
    check_output(case, out, ids, identity=True)
    # all experts local, weights renormalised: the layer returns its input
    np.testing.assert_allclose(out, case.inp["x"], rtol=0, atol=2e-6 * np.abs(case.inp["x"]).max())


def test_slot_permutation_is_bit_identical():
    wl = MoEWorkload(name="perm", tokens=400, **{**SMALL, "n_slots": 24})
    case = _case(wl)
    a = case.run()
    g = np.random.Generator(np.random.PCG64(5))
    case.place(g.permutation(24)[:16].astype(np.int32))
    b = case.run()
    np.testing.assert_array_equal(a, b)


def test_empty_token_batch_and_capacity_errors():
    from paper_2510_02613_amd import MoEError, MOE_ERR_CAPACITY, MOE_ERR_ARG
    wl = MoEWorkload(name="edge", tokens=64, **SMALL)
    case = _case(wl)
    out = case.layer.forward(case.x_dev[:0])
    assert out.shape[0] == 0
    with pytest.raises(MoEError) as ei:
        case.layer.forward(case.x_dev.repeat(2, 1))
    assert ei.value.status == MOE_ERR_CAPACITY
    with pytest.raises(MoEError) as ei:
        case.layer.forward(case.x_dev, shared_range=(0, 65))
    assert ei.value.status == MOE_ERR_ARG
    _full_check(case)  # the layer still works after rejected calls


def test_all_experts_remote_gives_zero_output():
    wl = MoEWorkload(name="remote", tokens=50, **SMALL)
    case = _case(wl, expert_map=np.full(16, -1, np.int32))
    out = case.run()
    assert (out == 0).all()
    v = case.layer.view(50)
    assert v["counts"].sum() == 0 and (v["inv"] == -1).all()


def test_shorter_batch_than_capacity_after_longer_one():
    wl = MoEWorkload(name="reuse", tokens=300, **SMALL)
    case = _case(wl)
    _full_check(case)
    _full_check(case, T=77)


# ---- the five benchmark configurations at full size ---------------------------

def test_qwen3_shape_full_size_all_tokens():
    case = _case(get_workload("qwen3_30b_a3b"))
    rep = {}
    _, v, err = _full_check(case, report=rep)
    assert v["offsets"][-1] == 4096 * 8 and rep["rows"] == 4096


def test_dsv3_rank_full_size_every_tile():
    """The largest configuration: 32 rows of every M-tile (36 chunks: whole rounds, the split last round, the
    four chunks of the shared expert) and 256 tokens of the whole batch are graded, over 1024 tokens in all."""
    case = _case(get_workload("dsv3_ep8_rank"))
    rep = {}
    _, v, _ = _full_check(case, sample=("tiles", 32, 256), report=rep)
    assert rep["rows"] >= 1024 and len(v["tiles"]) >= 36


def test_long_contraction_with_a_split_last_round():
    """288 one-chunk groups x one N-slice = 36 rows of 8 workgroups on a 32-row chip: the 4 rows of the last
    round have their contraction (H = 4096) shared out over 8 workgroups each and summed by a third launch.
    Every token is graded, so tiles of the whole rounds and of the split round are all covered."""
    wl = MoEWorkload(name="splitk", tokens=1800, hidden=4096, inter=64, n_experts=288, top_k=8, n_slots=288,
                     n_local=288, act_dtype="bf16", router_dtype="bf16", gate="softmax", seed=17)
    case = _case(wl)
    _, v, _ = _full_check(case)
    assert len(v["tiles"]) == 288 and v["counts"].min() > 0      # the launch shape the test is about
    assert wl.tokens * wl.top_k >= 48 * wl.n_slots               # ... on the large-tile kernels


def test_dsv2_lite_shape_full_size_all_tokens():
    """third model shape of the paper's evaluation: 64 experts, top-6, no renormalisation, 2 shared experts"""
    rep = {}
    _full_check(_case(get_workload("dsv2_lite")), report=rep)
    assert rep["rows"] == 4096


def test_dsv3_decode_all_tokens():
    case = _case(get_workload("dsv3_ep8_decode"))
    _, v, _ = _full_check(case)
    assert v["counts"][:32].max() <= 16


def test_relayout_switch_keeps_buffers_and_matches_oracle():
    import torch
    wl = get_workload("qwen3_relayout")
    map_a, map_b = relayout_maps(wl)
    case = _case(wl, expert_map=map_a)
    _full_check(case)                       # phase A, every token
    ptrs = (case.layer.w13.data_ptr(), case.layer.w2.data_ptr(), case.layer.workspace.data_ptr())
    free0, _ = torch.cuda.mem_get_info()
    alloc0 = torch.cuda.memory_stats()["allocation.all.allocated"]
    # copy experts 32..63 into their (shuffled) free slots, then flip the table
    for e in range(32, 64):
        case.layer.load_slot(int(map_b[e]), case.inp["w13_experts"][e], case.inp["w2_experts"][e])
    base_alloc = torch.cuda.memory_stats()["allocation.all.allocated"]
    case.place(map_b, upload=False)
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == base_alloc  # the switch allocates nothing
    assert ptrs == (case.layer.w13.data_ptr(), case.layer.w2.data_ptr(), case.layer.workspace.data_ptr())
    # the pool on the device now equals the pool the oracle was given
    from gpu_util import tensor_to_host
    np.testing.assert_array_equal(tensor_to_host(case.layer.w13[40:42]), case.w13_pool[40:42])
    _full_check(case)                       # phase B, every token
    assert alloc0 <= base_alloc


def test_plain_expert_kernels_on_bf16_layer():
    """The non-MFMA expert kernels stay correct for bf16 layers (debugging path)."""
    from paper_2510_02613_amd import MOE_FLAG_FORCE_GENERIC
    wl = MoEWorkload(name="generic", tokens=300, **SMALL)
    _full_check(_case(wl), flags=MOE_FLAG_FORCE_GENERIC)


def test_phase_timing_reports_every_phase():
    from paper_2510_02613_amd import binding as B
    wl = MoEWorkload(name="prof", tokens=300, **SMALL)
    case = _case(wl)
    B.moe_profile_enable(case.layer.handle, 1)
    for _ in range(3):
        case.run()
    for back in range(3):
        ms = B.moe_profile_read(case.layer.handle, back)
        assert len(ms) == 5 and all(0 <= v < 1000 for v in ms) and sum(ms) > 0
    with pytest.raises(B.MoEError):
        B.moe_profile_read(case.layer.handle, 3)
    # sampling: of the next 7 forwards the 1st, 4th and 7th are recorded
    B.moe_profile_enable(case.layer.handle, 3)
    for _ in range(7):
        case.run()
    for back in range(6):                       # 3 earlier + 3 sampled recordings
        assert sum(B.moe_profile_read(case.layer.handle, back)) > 0
    with pytest.raises(B.MoEError):
        B.moe_profile_read(case.layer.handle, 6)
    # one phase only: two events per recorded forward, the other phases read 0; earlier recordings are forgotten
    gemm1 = B.PHASE_NAMES.index("gemm1")
    B.moe_profile_select(case.layer.handle, gemm1)
    with pytest.raises(B.MoEError):
        B.moe_profile_read(case.layer.handle, 0)
    B.moe_profile_enable(case.layer.handle, 1)
    for _ in range(2):
        case.run()
    for back in range(2):
        ms = B.moe_profile_read(case.layer.handle, back)
        assert 0 < ms[gemm1] < 1000 and all(v == 0 for i, v in enumerate(ms) if i != gemm1)
    for bad in (-2, 5):
        with pytest.raises(B.MoEError):
            B.moe_profile_select(case.layer.handle, bad)
    B.moe_profile_select(case.layer.handle, -1)
    case.run()
    assert all(v > 0 for v in B.moe_profile_read(case.layer.handle, 0))
    B.moe_profile_enable(case.layer.handle, 0)
    _full_check(case)


@pytest.mark.parametrize("tokens", [200, 1000, 3000])
def test_large_tile_kernels_small_shapes(tokens):
    """Shapes whose contraction lengths are whole K-steps take the 8-wavefront kernels: groups of
    ~50, ~250 and ~750 rows exercise partial token tiles, odd tile counts and multi-chunk groups."""
    wl = MoEWorkload(name="big8", tokens=tokens, **{**SMALL, "inter": 128, "hidden": 320, "seed": 13})
    _full_check(_case(wl))


def test_large_tile_kernels_grouped_gate_shared_expert():
    wl = MoEWorkload(name="big8g", tokens=1500, hidden=256, inter=192, n_experts=32, top_k=4,
                     n_slots=9, n_local=8, act_dtype="bf16", router_dtype="bf16",
                     gate="sigmoid_group", n_group=4, topk_group=2, routed_scale=2.5, n_shared=1,
                     shared_range=(100, 1317), seed=14)
    _full_check(_case(wl))


@pytest.mark.parametrize("tokens", [3, 24])
def test_weight_streaming_kernels_small_shapes(tokens):
    """Decode-sized batches take the weight-streaming expert kernels: ragged K (264, 136 are not
    multiples of the 128-wide K chunk), a shared expert whose rows span two 16-row tiles, slots
    with no rows at all."""
    wl = MoEWorkload(name="decode_small", tokens=tokens, hidden=264, inter=136, n_experts=32, top_k=4,
                     n_slots=17, n_local=16, act_dtype="bf16", router_dtype="bf16",
                     gate="sigmoid_group", n_group=4, topk_group=2, routed_scale=2.5, n_shared=1,
                     shared_range=(min(2, tokens), min(22, tokens)), seed=15)
    case = _case(wl)
    _, v, _ = _full_check(case)
    assert (v["counts"] == 0).any()


@pytest.mark.parametrize("tokens", [300, 1000])
@pytest.mark.parametrize("router", ["f32", "bf16"])
def test_tiled_gate_kernel_small_shapes(tokens, router):
    """The LDS-tiled gate logits kernel (chosen by itself only for large batches) on ragged small ones:
    partial token blocks, fp32 router split into bf16 planes and bf16 router."""
    from paper_2510_02613_amd.binding import MOE_FLAG_GATE_TILED
    wl = MoEWorkload(name="tiled_gate", tokens=tokens, **{**SMALL, "router_dtype": router, "n_experts": 80, "n_slots": 80,
                                                           "n_local": 80, "seed": 16})
    _full_check(_case(wl), flags=MOE_FLAG_GATE_TILED)


def test_tiled_gate_kernel_ragged_contraction():
    """H = 264 is not a whole number of 64-wide K-steps: the tiled gate then stages through registers
    (zero-filled tail) instead of direct copies."""
    from paper_2510_02613_amd.binding import MOE_FLAG_GATE_TILED
    wl = MoEWorkload(name="tiled_gate_r", tokens=500, **{**SMALL, "hidden": 264, "seed": 19})
    _full_check(_case(wl), flags=MOE_FLAG_GATE_TILED)


def test_tiled_gate_kernel_grouped_sigmoid():
    from paper_2510_02613_amd.binding import MOE_FLAG_GATE_TILED
    wl = MoEWorkload(name="tiled_gate_g", tokens=700, hidden=256, inter=136, n_experts=160, top_k=4,
                     n_slots=21, n_local=20, act_dtype="bf16", router_dtype="bf16",
                     gate="sigmoid_group", n_group=8, topk_group=3, routed_scale=2.5, n_shared=1,
                     shared_range=(0, 700), seed=17)
    _full_check(_case(wl), flags=MOE_FLAG_GATE_TILED)


def test_large_tile_list_is_ordered_by_size():
    """Where the large-tile kernels run, chunks hold at most 320 rows and the list is ordered by their
    number of 32-row token tiles, largest first (the order the kernels deal to the XCDs); Zipf-skewed routing
    gives chunks of every size."""
    wl = MoEWorkload(name="big8z", tokens=4000, **{**SMALL, "inter": 128, "hidden": 320, "n_experts": 32, "n_slots": 32,
                                                   "n_local": 32, "zipf_s": 1.2, "seed": 18})
    case = _case(wl)
    _, v, _ = _full_check(case)
    tiles = v["tiles"]
    assert tiles[:, 2].max() <= 320 and len(tiles) > 40
    cls = (tiles[:, 2] + 31) // 32
    assert (np.diff(cls) <= 0).all()
    # within a size: by the first assignment (token, position) routed to the chunk's group -- a key that does not
    # depend on the slot the group's expert sits in -- then by row
    slot_of = case.expert_map[v["topk_ids"]].reshape(-1)
    first = np.full(wl.n_slots, np.iinfo(np.int64).max, np.int64)
    np.minimum.at(first, slot_of[slot_of >= 0], np.nonzero(slot_of >= 0)[0])
    for c in np.unique(cls):
        same = tiles[cls == c]
        assert (np.diff(first[same[:, 0]] * (1 << 20) + same[:, 1]) > 0).all()
    assert len(np.unique(cls)) >= 4


@pytest.mark.parametrize("experts", [576, 1024])
def test_many_experts_selection_paths(experts):
    """More than 512 experts: the top-k candidates no longer fit a wavefront's registers and the
    selection walks LDS instead; 1024 is the most the layer accepts."""
    wl = MoEWorkload(name="many_experts", tokens=150, hidden=128, inter=64, n_experts=experts, top_k=6,
                     n_slots=32, n_local=32, act_dtype="bf16", router_dtype="f32", gate="softmax", seed=20)
    _full_check(_case(wl))


def test_configuration_limits():
    """The largest gate the layer accepts: 1024 experts in 64 groups, 32 selected per token, 4 shared experts."""
    wl = MoEWorkload(name="limits", tokens=90, hidden=128, inter=64, n_experts=1024, top_k=32,
                     n_slots=68, n_local=64, act_dtype="bf16", router_dtype="bf16", gate="sigmoid_group",
                     n_group=64, topk_group=40, routed_scale=1.5, n_shared=4, shared_range=(5, 77), seed=23)
    _full_check(_case(wl))


@pytest.mark.parametrize("n_group,per,topk_group,top_k", [(3, 5, 2, 4), (6, 12, 4, 7), (5, 24, 3, 8), (12, 3, 7, 6)])
def test_group_counts_and_sizes_that_are_no_powers_of_two(n_group, per, topk_group, top_k):
    """The selection kernel shares a group's experts out over a power-of-two number of lanes and finds an
    expert's group by a shift when the group size allows it: group counts and sizes of every other kind take
    the general path (division, lanes past the last group idle)."""
    wl = MoEWorkload(name="odd_groups", tokens=210, hidden=192, inter=72, n_experts=n_group * per, top_k=top_k,
                     n_slots=n_group * per + 1, n_local=n_group * per, act_dtype="bf16", router_dtype="f32",
                     gate="sigmoid_group", n_group=n_group, topk_group=topk_group, routed_scale=1.5, n_shared=1,
                     seed=40 + n_group)
    _full_check(_case(wl))


def test_groups_of_one_expert():
    """n_group = E: every group is a single expert and its score is that expert's score alone; keeping the
    topk_group best groups and then the k best experts is plain top-k."""
    wl = MoEWorkload(name="group1", tokens=300, hidden=256, inter=136, n_experts=32, top_k=4,
                     n_slots=13, n_local=12, act_dtype="bf16", router_dtype="bf16",
                     gate="sigmoid_group", n_group=32, topk_group=9, routed_scale=1.5, n_shared=1,
                     shared_range=(20, 280), seed=24)
    case = _case(wl)
    _, v, _ = _full_check(case)
    plain = np.sort(np.argsort(-case.oracle_route()[3], axis=1, kind="stable")[:, :4], 1)
    flagged = case.oracle_route()[2] != 0
    np.testing.assert_array_equal(np.sort(v["topk_ids"], 1)[~flagged], plain[~flagged])


def _permuted_placement_is_bit_identical(wl, seed, expect_kernel):
    """The same layer with its experts in two different slot assignments (weights moved accordingly):
    outputs must agree bit for bit -- where an expert sits must not change any row's arithmetic."""
    case = _case(wl)
    a = case.run()
    v = case.layer.view(wl.tokens)
    expect_kernel(wl, v)
    g = np.random.Generator(np.random.PCG64(seed))
    n_routed = wl.n_slots - wl.n_shared
    slots = g.permutation(n_routed)[:min(wl.n_local, n_routed)].astype(np.int32)
    assert not np.array_equal(slots, np.arange(slots.size))
    case.place(block_expert_map(wl.n_experts, 0, slots.size, slots))
    b = case.run()
    np.testing.assert_array_equal(a, b)
    return case


def test_slot_permutation_bit_identical_large_tiles_multi_chunk_groups():
    """Large-tile kernels with Zipf-skewed groups of up to a dozen chunks: chunk order in the tile list moves
    with the placement, the rows' arithmetic must not."""
    wl = MoEWorkload(name="perm8", tokens=4000, **{**SMALL, "inter": 128, "hidden": 320, "n_experts": 32, "n_slots": 40,
                                                   "n_local": 32, "zipf_s": 1.2, "seed": 25})
    def expect(wl, v):
        assert wl.tokens * wl.top_k >= 48 * wl.n_slots and v["counts"].max() > 640
    _permuted_placement_is_bit_identical(wl, 6, expect)


def test_slot_permutation_bit_identical_weight_streaming_kernels():
    wl = MoEWorkload(name="permd", tokens=24, hidden=264, inter=136, n_experts=32, top_k=4,
                     n_slots=21, n_local=16, act_dtype="bf16", router_dtype="bf16",
                     gate="sigmoid_group", n_group=4, topk_group=2, routed_scale=2.5, n_shared=1,
                     shared_range=(2, 22), seed=26)
    def expect(wl, v):
        assert wl.tokens * wl.top_k <= 4 * wl.n_experts
    _permuted_placement_is_bit_identical(wl, 7, expect)


def test_slot_permutation_bit_identical_split_last_round():
    """H = 4096 on the large-tile kernels with a last round whose tiles' contractions are shared out over
    several workgroups: which tiles those are must not depend on the slots the experts sit in."""
    wl = MoEWorkload(name="perms", tokens=1800, hidden=4096, inter=64, n_experts=288, top_k=8, n_slots=300,
                     n_local=288, act_dtype="bf16", router_dtype="bf16", gate="softmax", seed=17)
    def expect(wl, v):
        assert len(v["tiles"]) == 288 and wl.tokens * wl.top_k >= 48 * wl.n_slots
    _permuted_placement_is_bit_identical(wl, 8, expect)


@pytest.mark.parametrize("experts", [16, 576])
def test_fewer_candidates_than_k_stays_in_bounds(experts):
    """A selection bias of -inf on all but two experts leaves a token two candidates for k = 4: the two are
    selected with their renormalised scores, the other two positions carry weight 0 and an id inside [0, E),
    and the output is the two experts' weighted sum (register and LDS selection paths)."""
    import oracle
    from gpu_util import to_f64, rel_err, TOL
    wl = MoEWorkload(name="few_candidates", tokens=150, **{**SMALL, "n_experts": experts, "hidden": 128, "inter": 64,
                                                             "n_slots": 16, "n_local": 16, "seed": 27})
    sb = np.full(experts, -np.inf, np.float32)
    sb[[2, 7]] = 0.0
    case = _case(wl, select_bias=sb)
    out = case.run()
    v = case.layer.view(wl.tokens)
    ids, w = v["topk_ids"], v["topk_w"]
    assert (ids >= 0).all() and (ids < experts).all()
    real = w != 0
    assert (real.sum(1) == 2).all()
    assert (np.sort(np.where(real, ids, -1), 1)[:, 2:] == [2, 7]).all()
    np.testing.assert_allclose(w.sum(1), 1.0, atol=1e-5)
    c = case.oracle_route()[3]                     # selection scores; experts 2 and 7 are un-biased
    s2, s7 = c[:, 2].astype(np.float64), c[:, 7].astype(np.float64)
    w2 = np.where((ids == 2) & real, w, 0).sum(1)
    np.testing.assert_allclose(w2, s2 / (s2 + s7), atol=1e-5)
    want = oracle.forward_routed(case.spec, case.inp["x"], case.w13_pool, case.w2_pool, case.expert_map,
                                 np.where(real, ids, -1).astype(np.int32), w)
    assert rel_err(to_f64(out), want) <= TOL["bf16"]


def test_largest_fp32_router_gate_tiling():
    """8192 tokens with an fp32 router: the gate logits run on the largest token x expert tiling of the
    direct-to-LDS kernel (128 x 128, rings for token and router rows); routing graded on every token."""
    wl = MoEWorkload(name="gate128", tokens=8192, hidden=256, inter=64, n_experts=128, top_k=4, n_slots=9,
                     n_local=8, act_dtype="bf16", router_dtype="f32", gate="softmax", seed=28)
    _full_check(_case(wl), sample=256)


def test_many_slots_bookkeeping():
    """A pool of 1500 slots (the scan over the slots takes several rounds in every bookkeeping kernel), 1024
    experts of which 900 are resident in scattered slots, 3 shared experts; both bookkeeping paths."""
    from paper_2510_02613_amd.binding import MOE_FLAG_PERMUTE_UNFUSED
    wl = MoEWorkload(name="many_slots", tokens=700, hidden=64, inter=8, n_experts=1024, top_k=8, n_slots=1500,
                     n_local=900, act_dtype="bf16", router_dtype="bf16", gate="softmax", n_shared=3,
                     shared_range=(13, 650), seed=29)
    g = np.random.Generator(np.random.PCG64(31))
    slots = g.permutation(1497)[:900].astype(np.int32)
    case = _case(wl, expert_map=block_expert_map(1024, 0, 900, slots))
    out, v, _ = _full_check(case)
    out2, v2, _ = _full_check(case, flags=MOE_FLAG_PERMUTE_UNFUSED)
    for key in ("counts", "offsets", "perm", "inv"):
        np.testing.assert_array_equal(v[key], v2[key])
    np.testing.assert_array_equal(out, out2)
    assert (v["counts"] > 0).sum() > 500


def test_tiles_of_a_slot_share_an_xcd():
    """Zipf-skewed routing on the large-tile kernels: hot experts have many tiles; the unit lists keep the tiles
    of a slot (of one size) in one column, i.e. on one XCD, for nearly all of them (a group larger than half a
    column is cut), and the lists still cover every tile and N-slice once (checked by check_bookkeeping)."""
    from gpu_util import check_units
    wl = MoEWorkload(name="colocate", tokens=6000, **{**SMALL, "inter": 1024, "hidden": 4096, "n_experts": 32, "n_slots": 32,
                                                     "n_local": 32, "zipf_s": 1.2, "seed": 30})
    case = _case(wl)
    _, v, _ = _full_check(case)
    shares = check_units(case, v)
    assert (v["counts"] > 640).sum() >= 3            # several slots with three or more tiles
    assert all(s is not None and s >= 0.7 for s in shares), shares


def test_shared_expert_tiles_share_an_xcd_on_the_dsv3_shape_small():
    """One shared expert over 1200 tokens beside single-tile experts (the shape of the DeepSeek-V3-style rank, scaled
    down): the shared slot's four tiles sit in one column of each unit list."""
    from gpu_util import check_units
    wl = MoEWorkload(name="colocate_shared", tokens=4800, hidden=4096, inter=1024, n_experts=128, top_k=8, n_slots=17,
                     n_local=16, act_dtype="bf16", router_dtype="bf16", gate="sigmoid_group", n_group=8, topk_group=4,
                     routed_scale=2.5, n_shared=1, shared_range=(0, 1200), seed=31)
    case = _case(wl)
    _, v, _ = _full_check(case)
    assert v["counts"][16] == 1200 and (v["tiles"][:, 0] == 16).sum() == 4
    whole = []
    shares = check_units(case, v, whole)
    assert shares == [1.0, 1.0], shares
    # every tile is two runs of N-slices here: the single tiles that fit under the even column height keep both
    # runs on one XCD (12 of 16), the rest even the columns out unit by unit
    assert all(w is not None and w >= 0.7 for w in whole), whole


@pytest.mark.parametrize("tokens", [1, 7, 16, 17, 40, 64])
@pytest.mark.parametrize("gate", ["softmax", "sigmoid_group"])
def test_few_tokens_expert_kernels_derive_their_tiles(tokens, gate):
    """Up to 64 tokens and 64 slots the weight-streaming GEMM-1 is launched without the offsets / permutation /
    tile-list kernel in front of it: its workgroups derive their tile from the selection kernel's block masks
    and one of them writes the tables.  Output and tables must match the oracle and -- bit for bit, on a
    workspace whose scratch part was overwritten with NaN patterns before each pass -- the separate
    bookkeeping kernels' pass, with remote experts, a shared expert on part of the batch and spare slots."""
    import torch
    from gpu_util import Case, tensor_to_host
    from paper_2510_02613_amd import binding as B
    kw = dict(n_group=4, topk_group=2, routed_scale=2.5) if gate == "sigmoid_group" else {}
    wl = MoEWorkload(name="few", tokens=tokens, hidden=320, inter=136, n_experts=64, top_k=4, n_slots=23, n_local=20,
                     act_dtype="bf16", router_dtype="bf16", gate=gate, n_shared=1, shared_range=(tokens // 2, tokens),
                     seed=71 + tokens, **kw)
    case = _case(wl)
    out, v, _ = _full_check(case)
    scratch = B.moe_workspace_view(case.layer.handle).topk_ids - case.layer.workspace.data_ptr()
    runs = []
    for flags in (0, B.MOE_FLAG_PERMUTE_UNFUSED, 0):
        case.layer.workspace[scratch:].fill_(0xff)
        runs.append((case.run(flags=flags), case.layer.view(tokens)))
    for o, vv in runs:
        np.testing.assert_array_equal(o, out)
        for key in ("counts", "offsets", "perm", "inv", "tiles", "h", "y"):
            np.testing.assert_array_equal(vv[key], v[key])


def test_ceiling_kernels_run():
    """The measuring-stick kernels of the benchmark (register-only MFMA loop, plain read, read in the large-tile
    kernels' weight-copy shape) run on small buffers and leave them untouched."""
    import torch
    from paper_2510_02613_amd import binding as B
    buf = torch.arange(6 * 256 * 512 // 4, dtype=torch.int32, device="cuda:0")   # 6 tiles of 256 rows x 512 bytes
    before = buf.clone()
    sink = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    s = torch.cuda.current_stream().cuda_stream
    assert B.moe_ceiling_mfma(64, 100, True, sink.data_ptr(), s) > 0
    B.moe_ceiling_stream(buf.data_ptr(), buf.numel() * 4, sink.data_ptr(), s)
    for nt in (False, True):
        B.moe_ceiling_tile_stream(buf.data_ptr(), 6, 512, nt, s)
    torch.cuda.synchronize()
    assert torch.equal(buf, before)
