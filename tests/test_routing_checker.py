"""The routing grader of the GPU tests (gpu_util.legal_selection) on the CPU: it must accept what the
ordering rule allows once fp32 scores closer than 1e-5 count as equal, and nothing else.  Mistakes are
planted here, on the CPU side, never on the GPU."""
import numpy as np

import oracle
from oracle import LayerSpec
from gpu_util import legal_selection, TIE, row_errors


def _route(T, E, k, G, KG, seed):
    g = np.random.Generator(np.random.PCG64(seed))
    x = g.standard_normal((T, E)).astype(np.float32)
    spec = LayerSpec(T=T, H=E, I=1, E=E, k=k, S=E, gate="sigmoid_group", n_group=G, topk_group=KG)
    ids, w, flags, c = oracle.route(spec, x, np.eye(E, dtype=np.float32), want_scores=True)
    return ids, flags, c


def test_oracle_selection_is_legal_and_planted_mistakes_are_not():
    T, E, k, G, KG = 300, 32, 4, 8, 3
    ids, flags, c = _route(T, E, k, G, KG, 3)
    per = E // G
    rejected_low = rejected_group = 0
    for t in range(T):
        assert legal_selection(c[t], ids[t], k, G, KG) is None
        if flags[t]:
            continue
        # swap the weakest chosen expert for a clearly worse one of a kept group
        kept = {int(e) // per for e in ids[t]}
        pool = [e for e in range(E) if e // per in kept and e not in ids[t] and c[t, e] < c[t, ids[t]].min() - 10 * TIE]
        if pool:
            bad = ids[t].copy()
            bad[-1] = pool[0]
            if len({int(e) // per for e in bad}) <= KG:
                # the left-out expert now beats a chosen one
                assert legal_selection(c[t], bad, k, G, KG) is not None
                rejected_low += 1
        # take the best expert of a group that clearly lost the group selection
        grp = np.sort(c[t].reshape(G, per), axis=1)
        gs = grp[:, -1] + grp[:, -2]
        g_th = np.sort(gs)[G - KG]
        losers = [q for q in range(G) if gs[q] < g_th - 10 * TIE]
        if losers:
            q = losers[0]
            bad = ids[t].copy()
            bad[0] = q * per + int(np.argmax(c[t, q * per:(q + 1) * per]))
            assert legal_selection(c[t], bad, k, G, KG) is not None
            rejected_group += 1
    assert rejected_low > 100 and rejected_group > 100


def test_group_near_tie_allows_either_group_and_only_its_best_experts():
    # 3 groups of 2, keep 1: group scores 1.0, 1.000004 (near-tie), 0.5
    c = np.array([0.6, 0.4, 0.7, 0.300004, 0.3, 0.2], np.float32)
    assert legal_selection(c, [2], 1, 3, 1) is None        # the rule's own choice: group 1 (higher score)
    assert legal_selection(c, [0], 1, 3, 1) is None        # group 0 is within 1e-5: legal
    assert legal_selection(c, [1], 1, 3, 1) is not None    # ... but not its second-best expert
    assert legal_selection(c, [4], 1, 3, 1) is not None    # group 2 is not near
    c2 = c.copy()
    c2[3] = 0.3001                                          # gap 1e-4: no near-tie any more
    assert legal_selection(c2, [0], 1, 3, 1) is not None
    assert legal_selection(c2, [2], 1, 3, 1) is None


def test_expert_near_tie_without_groups():
    c = np.array([0.5, 0.2, 0.200004, 0.1], np.float32)
    assert legal_selection(c, [0, 1], 2, 1, 1) is None
    assert legal_selection(c, [0, 2], 2, 1, 1) is None
    assert legal_selection(c, [0, 3], 2, 1, 1) is not None
    assert legal_selection(c, [1, 2], 2, 1, 1) is not None


def test_row_errors_use_each_rows_own_scale():
    want = np.array([[100.0, 1.0], [1.0, 0.5], [0.0, 0.0], [1e-6, 0.0]])
    got = want.copy()
    got[1, 0] += 0.05      # 5 % of ITS row's largest value, 0.05 % of the global one
    got[3, 0] += 1e-3      # a nearly-zero row is held to the floor (1e-3 * 100), not to its own 1e-6
    r = row_errors(got, want)
    np.testing.assert_allclose(r, [0.0, 0.05, 0.0, 1e-3 / 0.1], rtol=1e-12)
