"""The pass under HIP graph capture: it allocates nothing, never synchronises and contains no memset or
memcpy nodes, so a captured forward must replay, on new inputs and after a map switch, to exactly
what the eager path gives."""
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
