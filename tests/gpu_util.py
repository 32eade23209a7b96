"""Shared helpers of the GPU parity tests: build a layer from a seeded workload,
run it through the C ABI, and grade it against the CPU oracle."""
from __future__ import annotations

import numpy as np

import oracle
from oracle import LayerSpec
from workloads import (MoEWorkload, make_inputs, build_slot_pool, bf16_bits_to_f32,
                       block_expert_map, shared_slots_of)

TOL = {"bf16": 1e-2, "f32": 1e-4}   # max-relative-error bar on the layer output
W_ATOL = 1e-5                        # combine weights, times routed_scale
TIE = 1e-5                           # fp32 score gap under which a routing flip is legal


def to_f64(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


def tensor_to_host(t):
    a = t.detach().cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.int16 else a


class Case:
    """A workload instantiated on the GPU plus everything the oracle needs."""

    def __init__(self, wl: MoEWorkload, expert_map=None, shared_slots=None, inputs=None,
                 select_bias=None, max_tokens=None, pools=None):
        """pools = (w13 VirtualPool, w2 VirtualPool): the layer runs on those instead of plain allocations;
        then only the slots the placement uses are uploaded (the others may have no page under them)."""
        from paper_2510_02613_amd.layer import MoELayer
        self.wl = wl
        self.inp = make_inputs(wl) if inputs is None else inputs
        self.spec = LayerSpec.from_workload(wl)
        self.expert_map = (block_expert_map(wl.n_experts, 0, min(wl.n_local, wl.n_slots - wl.n_shared))
                           if expert_map is None else np.asarray(expert_map, np.int32))
        self.shared_slots = shared_slots_of(wl) if shared_slots is None else np.asarray(shared_slots, np.int32)
        self.select_bias = select_bias
        self.layer = MoELayer(hidden=wl.hidden, inter=wl.inter, n_experts=wl.n_experts, top_k=wl.top_k,
                              n_slots=wl.n_slots, max_tokens=max_tokens or max(wl.tokens, 1),
                              act_dtype=wl.act_dtype, router_dtype=wl.router_dtype, gate=wl.gate,
                              n_group=wl.n_group, topk_group=wl.topk_group, renormalize=wl.renormalize,
                              routed_scale=wl.routed_scale, n_shared=wl.n_shared,
                              router_w=self.inp["router_w"], logit_bias=self.inp["logit_bias"],
                              select_bias=select_bias, **({} if pools is None else dict(w13_pool=pools[0], w2_pool=pools[1])))
        if pools is None:
            self.place(self.expert_map, self.shared_slots)
        else:
            self.place(self.expert_map, self.shared_slots, upload=False)
            for s in sorted(set(int(v) for v in self.expert_map if v >= 0) | set(int(v) for v in self.shared_slots[:wl.n_shared])):
                self.layer.load_slot(s, self.w13_pool[s], self.w2_pool[s])
        self.x_dev = self.layer.upload(self.inp["x"])

    def place(self, expert_map, shared_slots=None, upload=True):
        """(Re)build the slot pools for a placement and install the map."""
        wl = self.wl
        self.expert_map = np.asarray(expert_map, np.int32)
        if shared_slots is not None:
            self.shared_slots = np.asarray(shared_slots, np.int32)
        self.w13_pool = build_slot_pool(self.inp["w13_experts"], self.expert_map, wl.n_slots, wl.n_local, self.shared_slots)
        self.w2_pool = build_slot_pool(self.inp["w2_experts"], self.expert_map, wl.n_slots, wl.n_local, self.shared_slots)
        if upload:
            self.layer.load_pool(self.w13_pool, self.w2_pool)
        self.layer.set_expert_map(self.expert_map, self.shared_slots if wl.n_shared else None)

    def run(self, flags=0, T=None, shared_range=None):
        import torch
        T = self.wl.tokens if T is None else T
        sr = self.wl.shared_range if shared_range is None else shared_range
        out = self.layer.forward(self.x_dev[:T], shared_range=sr, flags=flags)
        torch.cuda.synchronize()
        return tensor_to_host(out)

    # ---- oracle side ---------------------------------------------------------
    def oracle_route(self):
        return oracle.route(self.spec, self.inp["x"], self.inp["router_w"], self.inp["logit_bias"],
                            self.select_bias, want_scores=True)

    def oracle_forward(self, tokens=None, forced_ids=None, identity=False, shared_range=None):
        sr = self.wl.shared_range if shared_range is None else shared_range
        return oracle.forward(self.spec, self.inp["x"], self.inp["router_w"], self.w13_pool, self.w2_pool,
                              self.expert_map, logit_bias=self.inp["logit_bias"], select_bias=self.select_bias,
                              shared_slots=self.shared_slots, shared_range=sr, tokens=tokens,
                              forced_ids=forced_ids, identity_experts=identity)


def legal_selection(c_t: np.ndarray, ids: np.ndarray, k: int, n_group: int, topk_group: int):
    """Is `ids` a selection the ordering rule allows for selection scores c_t once fp32 scores
    closer than TIE count as equal?  Returns None when it is, else a sentence saying why not.

    Groups (n_group > 1): a group's score is the fp32 sum of its two largest scores (its largest,
    for groups of one).  With g_th the topk_group-th largest group score, a kept-group set is
    legal when it holds every group scoring >= g_th + TIE, and otherwise only groups within TIE
    of g_th, topk_group groups in all.  Inside a legal kept set the k ids must be its best
    experts up to near-ties: no expert left out may beat a chosen one by TIE or more."""
    import itertools
    E = c_t.shape[0]
    ids = [int(e) for e in ids]
    if n_group > 1:
        per = E // n_group
        grp = np.sort(c_t.reshape(n_group, per), axis=1)
        gs = (grp[:, -1] + grp[:, -2]).astype(np.float32) if per > 1 else grp[:, -1].copy()
        g_th = np.sort(gs)[n_group - topk_group]
        sure = [g for g in range(n_group) if gs[g] >= g_th + np.float32(TIE)]
        near = [g for g in range(n_group) if abs(float(gs[g]) - float(g_th)) < TIE]
        used = {e // per for e in ids}
        stray = used - set(sure) - set(near)
        if stray:
            return f"ids come from groups {sorted(stray)} whose scores are not within {TIE} of the {topk_group}-th group score"
        need = topk_group - len(sure)
        options = [set(sure) | set(extra) for extra in itertools.combinations(near, need)] if 0 <= need <= len(near) else []
        options = [K for K in options if used <= K]
        if not options:
            return f"groups {sorted(used)} fit no legal kept-group set (sure {sure}, near-tied {near})"
    else:
        per = E
        options = [{0}]
    why = None
    for K in options:
        members = np.array([e for e in range(E) if e // per in K])
        chosen = np.zeros(E, bool)
        chosen[ids] = True
        left = members[~chosen[members]]
        if left.size == 0:
            return None
        worst_in = float(c_t[ids].min())
        best_out = float(c_t[left].max())
        if best_out - worst_in < TIE:
            return None
        why = (f"expert {int(left[np.argmax(c_t[left])])} (score {best_out}) was left out although it beats "
               f"a chosen one (score {worst_in}) by {best_out - worst_in:.3g}")
    return why


def check_routing(case: Case, gpu_ids: np.ndarray, gpu_w: np.ndarray):
    """Routing parity: identical expert sets on every unflagged token; on a flagged token
    (expert near-tie, group near-tie, or both) a different set must still be a selection the
    ordering rule allows when fp32 scores closer than TIE count as equal (legal_selection).
    Weights agree to W_ATOL * scale per expert.  Returns (ids to grade the output with,
    number of flagged tokens, number of legal flips)."""
    o_ids, o_w, flags, c = case.oracle_route()
    T, k = o_ids.shape
    wl = case.wl
    assert gpu_ids.shape == (T, k)
    assert (gpu_ids >= 0).all() and (gpu_ids < wl.n_experts).all()
    srt_g, srt_o = np.sort(gpu_ids, 1), np.sort(o_ids, 1)
    assert (np.diff(srt_g, axis=1) > 0).all(), "a token selected the same expert twice"
    differ = (srt_g != srt_o).any(1)
    bad = differ & (flags == 0)
    assert not bad.any(), f"routing differs on unflagged tokens {np.nonzero(bad)[0][:8]}"
    grouped = wl.gate == "sigmoid_group" and wl.n_group > 1
    flips = 0
    for t in np.nonzero(differ)[0]:
        why = legal_selection(c[t], gpu_ids[t], k, wl.n_group if grouped else 1, wl.topk_group if grouped else 1)
        assert why is None, f"token {t} (flags {int(flags[t])}): {why}"
        flips += 1
    # weights, matched per expert id (positions may differ among near-equal scores)
    scale = abs(wl.routed_scale)
    same = ~differ
    og = np.argsort(gpu_ids, 1)
    oo = np.argsort(o_ids, 1)
    wg = np.take_along_axis(gpu_w.astype(np.float64), og, 1)
    wo = np.take_along_axis(o_w, oo, 1)
    err = np.abs(wg - wo)[same]
    assert err.max(initial=0.0) <= W_ATOL * scale, f"weight error {err.max()}"
    return gpu_ids, int((flags != 0).sum()), flips


def ran_large_tiles(wl, T, flags=0):
    """Did a pass of T tokens run the large-tile expert kernels (the host's rule, from shapes alone)?"""
    return (wl.act_dtype == "bf16" and wl.hidden % 64 == 0 and wl.inter % 64 == 0 and not (flags & 3)
            and T * (wl.top_k + wl.n_shared) >= 48 * wl.n_slots)


def check_bookkeeping(case: Case, v: dict, T: int, shared_range, flags=0):
    """counts / offsets / perm / inv against their definitions, from the GPU's own ids; the tile list; and,
    after a pass on the large-tile kernels, their work-unit lists."""
    wl = case.wl
    k, kk, S = wl.top_k, wl.top_k + wl.n_shared, wl.n_slots
    ids = v["topk_ids"]
    slot = np.full((T, kk), -1, np.int64)
    slot[:, :k] = case.expert_map[ids]
    for i in range(wl.n_shared):
        slot[shared_range[0]:shared_range[1], k + i] = case.shared_slots[i]
    np.testing.assert_array_equal(v["active_map"], np.concatenate([case.expert_map, case.shared_slots[:wl.n_shared]]))
    counts = np.bincount(slot[slot >= 0], minlength=S)
    np.testing.assert_array_equal(v["counts"], counts)
    np.testing.assert_array_equal(v["offsets"], np.concatenate([[0], np.cumsum(counts)]))
    A = int(counts.sum())
    inv = v["inv"]
    np.testing.assert_array_equal(inv >= 0, slot >= 0)
    rows = inv[inv >= 0]
    assert rows.size == A and np.array_equal(np.sort(rows), np.arange(A)), "inv is not a bijection onto [0,A)"
    tok = np.repeat(np.arange(T)[:, None], kk, 1)
    np.testing.assert_array_equal(v["perm"][rows], tok[inv >= 0])
    offs = v["offsets"]
    s_of_row = np.searchsorted(offs, rows, side="right") - 1
    np.testing.assert_array_equal(s_of_row, slot[inv >= 0])
    # rows of one slot are ordered by (token, position): deterministic layout
    for s in range(S):
        r = inv[slot == s]
        assert (np.diff(r) > 0).all()
    # the M-tile list of the expert kernels: every grouped row in exactly one tile of its own slot
    tiles = v["tiles"]
    if A:
        assert (tiles[:, 2] > 0).all()
        # fourth field: 1 exactly when the tile is all of its slot's rows
        np.testing.assert_array_equal(tiles[:, 3], (tiles[:, 2] == counts[tiles[:, 0]]).astype(np.int32))
        covered = np.zeros(A, np.int32)
        for s_, r0, n, _ in tiles:
            assert offs[s_] <= r0 and r0 + n <= offs[s_ + 1], "a tile leaves its slot's rows"
            covered[r0:r0 + n] += 1
        assert (covered == 1).all(), "tiles do not partition the grouped rows"
    else:
        assert len(tiles) == 0
    if A and ran_large_tiles(wl, T, flags):
        check_units(case, v)


def check_units(case: Case, v: dict, whole=None):
    """The work-unit lists of the large-tile kernels (call after a pass that ran them): per GEMM, every N-slice
    of every tile is in exactly one unit, holes only at the ends of the eight columns, columns differ by at most
    a few units, and the tiles of a slot that sit together in the tile list share a column when the pass has
    such groups.  Returns, per GEMM, the share of the avoidable weight fetches (tiles - 1 per multi-tile slot and
    size) that the columns avoid; whole (a list) receives, per GEMM, the share of the single tiles whose runs sit
    in one column."""
    wl = case.wl
    tiles, hdr, lists = v["tiles"], v["unit_hdr"], v["units"]
    n_slices = ((wl.inter + 127) // 128, (wl.hidden + 255) // 256)
    shares = []
    for w in range(2):
        n_rows, spp, n_units, runs = (int(x) for x in hdr[w])
        u = lists[w]
        assert len(u) == n_units and n_units % 8 == 0 and n_rows == n_units // 8 * spp and spp * runs == n_slices[w]
        live = u[:, 2] > 0
        cols = np.arange(n_units) % 8
        for x in range(8):                                   # a column's holes are all at its end
            lx = live[cols == x]
            assert not (np.diff(lx.astype(np.int8)) > 0).any(), "a hole inside a column"
        fills = np.array([live[cols == x].sum() for x in range(8)])
        assert fills.max() - fills.min() <= 3 or len(tiles) * runs < 16, fills
        seen = {}
        for slot, r0, rows, info in u[live]:
            s0 = info >> 1
            assert s0 % spp == 0 and s0 + spp <= n_slices[w]
            seen[(int(slot), int(r0), int(rows), int(info & 1), int(s0))] = seen.get((int(slot), int(r0), int(rows), int(info & 1), int(s0)), 0) + 1
        want = {(int(s_), int(r0), int(n), int(f), r * spp) for s_, r0, n, f in tiles for r in range(runs)}
        assert set(seen) == want and all(c == 1 for c in seen.values()), "units do not cover every (tile, run) exactly once"
        # co-location: tiles of one slot and one size class (32-row tiles) in one column, run by run
        groups = {}
        for i in np.nonzero(live)[0]:
            slot, r0, rows, info = u[i]
            groups.setdefault((int(slot), (int(rows) + 31) // 32, int(info >> 1)), set()).add(int(cols[i]))
        sizes = {}
        for slot, r0, rows, info in u[live]:
            sizes[(int(slot), (int(rows) + 31) // 32, int(info >> 1))] = sizes.get((int(slot), (int(rows) + 31) // 32, int(info >> 1)), 0) + 1
        multi = [k for k, c in sizes.items() if c > 1]
        # of the weight fetches that sharing a column can save (tiles - 1 per group), the share that is saved
        # (tiles - columns used); groups larger than half a column are cut on purpose
        shares.append(sum(sizes[k] - len(groups[k]) for k in multi) / sum(sizes[k] - 1 for k in multi) if multi else None)
        if whole is not None:
            # of the tiles that are alone in their slot, the share whose runs all sit in ONE column (their token
            # rows are then fetched by one XCD); None when tiles are not split into runs
            per_tile = {}
            for i in np.nonzero(live)[0]:
                slot, r0, rows, info = u[i]
                per_tile.setdefault((int(slot), int(r0)), set()).add(int(cols[i]))
            alone = [k for k in per_tile if sum(1 for q in per_tile if q[0] == k[0]) == 1]
            whole.append(sum(len(per_tile[k]) == 1 for k in alone) / len(alone) if runs > 1 and alone else None)
    return shares


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max |got - want| / max |want| over the whole array."""
    den = np.abs(want).max()
    if den == 0:
        return float(np.abs(got).max())
    return float(np.abs(got - want).max() / den)


ROW_FLOOR = 1e-3   # a row's own scale counts down to this fraction of the largest reference magnitude


def row_errors(got: np.ndarray, want: np.ndarray) -> np.ndarray:
    """Per row: max |got - want| over the row / max |want| over THE ROW, the denominator floored at
    ROW_FLOOR * max |want| over everything (a row that is almost zero is not held to its own scale)."""
    if want.size == 0:
        return np.zeros(0)
    floor = ROW_FLOOR * np.abs(want).max()
    den = np.maximum(np.abs(want).max(1), floor)
    den[den == 0] = 1.0
    return np.abs(got - want).max(1) / den


def check_output(case: Case, out_bits: np.ndarray, grade_ids: np.ndarray, tokens=None, identity=False,
                 shared_range=None, report=None):
    """Layer output against the fp64 oracle: the max-relative-error bar over all compared rows, and the
    same bar row by row against each row's own largest reference magnitude.  report: a dict that
    receives the two figures and the worst row."""
    want = case.oracle_forward(tokens=tokens, forced_ids=grade_ids, identity=identity, shared_range=shared_range)
    got = to_f64(out_bits if tokens is None else out_bits[np.asarray(tokens)])
    assert np.isfinite(got).all()
    err = rel_err(got, want)
    tol = TOL[case.wl.act_dtype]
    assert err <= tol, f"max relative error {err:.3e} > {tol}"
    # rows whose reference is all zero must be exactly zero
    zero = np.abs(want).max(1) == 0 if want.size else np.zeros(0, bool)
    assert (got[zero] == 0).all()
    rows = row_errors(got, want)
    worst = int(np.argmax(rows)) if rows.size else -1
    worst_tok = worst if tokens is None or worst < 0 else int(np.asarray(tokens)[worst])
    print(f"[{case.wl.name}] rows graded {rows.size}  max rel err {err:.3e}  worst row: token {worst_tok} "
          f"row err {rows.max(initial=0.0):.3e}", flush=True)
    if report is not None:
        report.update(rows=int(rows.size), err=err, worst_row_err=float(rows.max(initial=0.0)), worst_token=worst_tok)
    assert rows.max(initial=0.0) <= tol, f"token {worst_tok}: row error {rows.max():.3e} > {tol}"
    return err
