"""The pass under HIP graph capture: it allocates nothing, never synchronises and contains no memset or
memcpy nodes, so a captured forward must replay, on new inputs, to exactly what the eager path gives --
and, since the expert table sits at one fixed address, also after map switches and slot fills that
happen between replays of a graph captured before them."""
import numpy as np
import pytest

from workloads import MoEWorkload

pytestmark = pytest.mark.gpu

SHAPES = {
    "large_tile": dict(tokens=900, hidden=320, inter=128, n_experts=16, top_k=4, n_slots=16, n_local=16,
                       act_dtype="bf16", router_dtype="f32", gate="softmax", seed=51),
    "weight_streaming": dict(tokens=24, hidden=264, inter=136, n_experts=32, top_k=4, n_slots=17, n_local=16,
                             act_dtype="bf16", router_dtype="bf16", gate="sigmoid_group", n_group=4, topk_group=2,
                             routed_scale=2.5, n_shared=1, shared_range=(2, 22), seed=52),
    "f32": dict(tokens=200, hidden=136, inter=72, n_experts=8, top_k=2, n_slots=8, n_local=8,
                act_dtype="f32", router_dtype="f32", gate="softmax", seed=53),
}


@pytest.mark.parametrize("shape", sorted(SHAPES))
def test_captured_forward_replays_like_eager(shape):
    import torch
    from gpu_util import Case, tensor_to_host
    wl = MoEWorkload(name="graph_" + shape, **SHAPES[shape])
    case = Case(wl)
    x = case.x_dev
    out = torch.empty_like(x)
    # three input batches: the seeded one, a permutation of its rows, and a scaled copy
    perm = torch.randperm(wl.tokens, generator=torch.Generator().manual_seed(5)).to(x.device)
    xs = [x.clone(), x[perm].clone()]
    xs.append((x.view(torch.bfloat16).float() * 0.5).to(torch.bfloat16).view(torch.int16) if wl.act_dtype == "bf16" else x * 0.5)
    eager = []
    for xi in xs:
        eager.append(tensor_to_host(case.layer.forward(xi, shared_range=wl.shared_range)))
    torch.cuda.synchronize()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        case.layer.forward(x, out=out, shared_range=wl.shared_range)        # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        case.layer.forward(x, out=out, shared_range=wl.shared_range)
    for rep in range(2):
        for xi, want in zip(xs, eager):
            x.copy_(xi)                      # eager work and a synchronisation between the replays
            graph.replay()
            torch.cuda.synchronize()
            np.testing.assert_array_equal(tensor_to_host(out), want)


def test_captured_forward_follows_map_switches_and_slot_fills():
    """One graph, captured under placement A.  Between its replays the placement is switched (A -> B -> C,
    twice over the same table address), with experts copied into free slots by background fills before
    the switch that starts using them; every replay must equal an eager pass under the placement in force."""
    import torch
    from gpu_util import Case, tensor_to_host
    from workloads import block_expert_map
    wl = MoEWorkload(name="graph_switch", tokens=900, hidden=320, inter=128, n_experts=16, top_k=4, n_slots=24,
                     n_local=16, act_dtype="bf16", router_dtype="f32", gate="softmax", seed=54)
    map_a = block_expert_map(16, 0, 8)                                  # experts 0..7 in slots 0..7
    case = Case(wl, expert_map=map_a)
    layer, x = case.layer, case.x_dev
    out = torch.empty_like(x)
    g = np.random.Generator(np.random.PCG64(3))
    map_b = map_a.copy()
    map_b[8:16] = 8 + g.permutation(16)[:8]                             # experts 8..15 join, in free slots 8..23
    map_c = np.full(16, -1, np.int32)
    map_c[8:16] = map_b[8:16]                                           # experts 0..7 leave

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        layer.forward(x, out=out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        layer.forward(x, out=out)

    def both():
        want = tensor_to_host(layer.forward(x))                          # eager, placement in force
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(tensor_to_host(out), want)
        return want

    a = both()
    copy = torch.cuda.Stream()
    serve = torch.cuda.current_stream()
    staged = [(layer.upload(case.inp["w13_experts"][e]), layer.upload(case.inp["w2_experts"][e])) for e in range(8, 16)]
    torch.cuda.synchronize()                                             # the sources are in place (and stay alive below)
    for e in range(8, 16):                                               # background fills into free slots
        layer.load_expert_async(int(map_b[e]), staged[e - 8][0], staged[e - 8][1], copy, serve)
    layer.set_expert_map(map_b)                                          # waits for the fills on the stream
    b = both()
    assert not np.array_equal(a, b)
    layer.set_expert_map(map_c)
    c = both()
    assert not np.array_equal(b, c)
    # the oracle agrees with the last placement (weights: slots 8..23 as filled, slots 0..7 as before)
    from gpu_util import check_routing, check_output
    case.expert_map = map_c
    from workloads import build_slot_pool
    case.w13_pool = build_slot_pool(case.inp["w13_experts"], map_b, wl.n_slots, wl.n_local, ())
    case.w2_pool = build_slot_pool(case.inp["w2_experts"], map_b, wl.n_slots, wl.n_local, ())
    v = layer.view(wl.tokens)
    ids, _, _ = check_routing(case, v["topk_ids"], v["topk_w"])
    check_output(case, c, ids)
