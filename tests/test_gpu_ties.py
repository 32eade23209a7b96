"""Exact ties in the selection: experts with IDENTICAL router rows get bit-identical logits on both sides, so
the rule "among equal scores the lower expert index wins" decides, and the GPU must take the oracle's choice."""
import numpy as np
import pytest

from workloads import MoEWorkload, make_inputs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("E,k,T,gate,act", [
    (128, 8, 300, "softmax", "bf16"),          # two candidates per lane
    (256, 8, 300, "sigmoid_group", "bf16"),    # four per lane, group limited
    (512, 6, 200, "softmax", "bf16"),          # eight per lane
    (576, 4, 100, "softmax", "bf16"),          # candidates in LDS
    (24, 3, 150, "softmax", "f32"),            # the fp32 gate
])
def test_equal_scores_go_to_the_lower_expert_index(E, k, T, gate, act):
    from gpu_util import Case, check_routing
    grouped = gate == "sigmoid_group"
    wl = MoEWorkload(name=f"ties{E}", tokens=T, hidden=128, inter=64, n_experts=E, top_k=k, n_slots=E, n_local=E,
                     act_dtype=act, router_dtype="f32", gate=gate, n_group=8 if grouped else 1,
                     topk_group=4 if grouped else 1, routed_scale=2.5 if grouped else 1.0, seed=31)
    inp = make_inputs(wl)
    # copies of router rows: the neighbour (another lane), 64 further (same lane, next register), far away
    r = inp["router_w"]
    g = np.random.Generator(np.random.PCG64(7))
    pairs = []
    for src in g.choice(E, size=E // 3, replace=False):
        for d in (1, 64, 193):
            dst = (int(src) + d) % E
            if grouped and dst // (E // 8) != int(src) // (E // 8):
                continue                      # keep group scores apart: ties inside a group only
            pairs.append((int(src), dst))
            break
    for src, dst in pairs:
        r[dst] = r[src]
    case = Case(wl, inputs=inp)
    case.run()
    v = case.layer.view(T)
    o_ids, _, flags, c = case.oracle_route()
    # how often the rule decided: the last selected and the first rejected score are EQUAL
    srt = -np.sort(-c, axis=1)
    decided = int((srt[:, k - 1] == srt[:, k]).sum()) if not grouped else None
    # tokens whose only near-ties are exact ties must match the oracle's ids exactly, in order
    exact_only = np.ones(T, bool)
    for t in range(T):
        d = np.abs(np.diff(srt[t, :min(E, 4 * k)]))
        exact_only[t] = not ((d > 0) & (d < 1e-5)).any()
    if not grouped:
        np.testing.assert_array_equal(v["topk_ids"][exact_only], o_ids[exact_only])
        assert decided > 0 or E < 64, "the case never exercised the rule at the selection boundary"
    check_routing(case, v["topk_ids"], v["topk_w"])      # the general bar, all tokens
    # equal scores inside the selection: positions follow the index order too
    same = (np.sort(v["topk_ids"], 1) == np.sort(o_ids, 1)).all(1)
    assert same.mean() > 0.95
