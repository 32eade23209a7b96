"""moe_forward_static -- the pass with every intermediate in the library's own device array, for callers that
cannot allocate -- against moe_forward on a layer of the same configuration and placement: bit-identical
outputs, on two calls in a row, the second with a smaller input (the array keeps the first call's contents)."""
import numpy as np
import pytest

from workloads import MoEWorkload

pytestmark = pytest.mark.gpu

SHAPES = {
    # large-tile kernels, fp32 router
    "large_tile": dict(tokens=900, hidden=320, inter=128, n_experts=16, top_k=4, n_slots=16, n_local=16,
                       act_dtype="bf16", router_dtype="f32", gate="softmax", seed=61),
    # weight-streaming kernels, grouped sigmoid gate, shared expert, experts of other ranks
    "weight_streaming": dict(tokens=24, hidden=264, inter=136, n_experts=32, top_k=4, n_slots=17, n_local=16,
                             act_dtype="bf16", router_dtype="bf16", gate="sigmoid_group", n_group=4, topk_group=2,
                             routed_scale=2.5, n_shared=1, shared_range=(2, 22), seed=62),
    # 128 x 128 kernels
    "mid": dict(tokens=300, hidden=256, inter=136, n_experts=16, top_k=4, n_slots=16, n_local=16,
                act_dtype="bf16", router_dtype="f32", gate="softmax", seed=63),
    "f32": dict(tokens=200, hidden=136, inter=72, n_experts=8, top_k=2, n_slots=8, n_local=8,
                act_dtype="f32", router_dtype="f32", gate="softmax", seed=64),
}


@pytest.mark.parametrize("shape", sorted(SHAPES))
def test_static_scratch_pass_equals_workspace_pass_twice_in_a_row(shape):
    import torch
    from gpu_util import Case, tensor_to_host, check_routing, check_output
    wl = MoEWorkload(name="static_" + shape, **SHAPES[shape])
    case = Case(wl)
    layer, x = case.layer, case.x_dev
    T1, T2 = wl.tokens, max(1, wl.tokens // 3)
    sr1 = wl.shared_range
    sr2 = (min(sr1[0], T2), min(sr1[1], T2))
    free0, _ = torch.cuda.mem_get_info()
    alloc0 = torch.cuda.memory_stats()["allocation.all.allocated"]
    out1 = torch.empty_like(x)
    out2 = torch.empty_like(x[:T2])
    alloc1 = torch.cuda.memory_stats()["allocation.all.allocated"]
    layer.forward_static(x, out=out1, shared_range=sr1)                 # first call: the full batch
    layer.forward_static(x[:T2], out=out2, shared_range=sr2)            # second call, smaller, right behind it
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == alloc1     # torch allocated nothing for the calls
    got1, got2 = tensor_to_host(out1), tensor_to_host(out2)
    want1 = tensor_to_host(layer.forward(x, shared_range=sr1))
    want2 = tensor_to_host(layer.forward(x[:T2], shared_range=sr2))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got1, want1)
    np.testing.assert_array_equal(got2, want2)
    # ... and the workspace pass it is compared with meets the oracle
    case.run()
    v = layer.view(wl.tokens)
    ids, _, _ = check_routing(case, v["topk_ids"], v["topk_w"])
    check_output(case, got1, ids)


def test_static_scratch_pass_rejects_what_does_not_fit():
    from paper_2510_02613_amd import binding as B
    from paper_2510_02613_amd import MoEError
    import torch
    cfg = B.MoEConfig(hidden=2048, inter=768, n_experts=128, top_k=8, n_slots=128, max_tokens=4096, act_dtype=B.MOE_BF16,
                      router_dtype=B.MOE_F32, gate=B.MOE_GATE_SOFTMAX_TOPK, n_group=1, topk_group=1, renormalize=1,
                      routed_scale=1.0, n_shared=0)
    d = torch.zeros(64, dtype=torch.int16, device="cuda")
    buf = B.MoEBuffers(d.data_ptr(), 0, 0, d.data_ptr(), d.data_ptr(), 0, 0)
    with pytest.raises(MoEError) as ei:   # 4096 tokens of this shape need ~190 MB of intermediates
        B.moe_forward_static(cfg, buf, list(range(128)), None, d.data_ptr(), 4096, d.data_ptr())
    assert ei.value.status == B.MOE_ERR_CAPACITY
    with pytest.raises(MoEError) as ei:   # a placement that claims a slot twice, on a pass that would fit
        B.moe_forward_static(cfg, buf, [0] * 128, None, d.data_ptr(), 16, d.data_ptr())
    assert ei.value.status == B.MOE_ERR_MAP
