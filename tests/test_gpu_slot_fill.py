"""Background slot fill (moe_load_expert) beside running forwards, then the map switch:
forwards before the switch are undisturbed, forwards after it match the oracle on the new placement."""
import numpy as np
import pytest

from workloads import MoEWorkload, relayout_maps

pytestmark = pytest.mark.gpu

MID = dict(hidden=512, inter=264, n_experts=32, top_k=4, n_slots=16, n_local=16,
           act_dtype="bf16", router_dtype="f32", gate="softmax", seed=31)


def test_fill_beside_forwards_then_switch():
    import torch
    from gpu_util import Case, tensor_to_host, check_routing, check_bookkeeping, check_output
    wl = MoEWorkload(name="fill", tokens=900, **MID)
    map_a, map_b = relayout_maps(wl)                     # phase A: experts 0..7 in slots 0..7; B adds 8..15 shuffled
    case = Case(wl, expert_map=map_a)
    dev = case.x_dev.device
    serve = torch.cuda.current_stream(dev)
    copy = torch.cuda.Stream(device=dev)
    before = case.run()
    # sources staged on the device (the landing buffers of a peer transfer)
    src = {e: (case.layer.upload(case.inp["w13_experts"][e]), case.layer.upload(case.inp["w2_experts"][e]))
           for e in range(8, 16)}
    torch.cuda.synchronize()
    alloc0 = torch.cuda.memory_stats()["allocation.all.allocated"]
    outs = []
    for e in range(8, 16):
        outs.append(case.layer.forward(case.x_dev, shared_range=wl.shared_range))           # serving goes on ...
        case.layer.load_expert_async(int(map_b[e]), src[e][0], src[e][1], copy, serve, copy_blocks=8)  # ... beside the fill
    outs.append(case.layer.forward(case.x_dev, shared_range=wl.shared_range))
    case.place(map_b, upload=False)                      # switch: waits (on the stream) for all eight fills
    after = case.layer.forward(case.x_dev, shared_range=wl.shared_range)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == alloc0 + len(outs) + 1   # only the output tensors
    for o in outs:                                       # forwards under the old map never saw the fills
        np.testing.assert_array_equal(tensor_to_host(o), before)
    np.testing.assert_array_equal(tensor_to_host(case.layer.w13), case.w13_pool)             # the pool is the new placement's
    np.testing.assert_array_equal(tensor_to_host(case.layer.w2), case.w2_pool)
    v = case.layer.view(wl.tokens)
    ids, _, _ = check_routing(case, v["topk_ids"], v["topk_w"])
    check_bookkeeping(case, v, wl.tokens, wl.shared_range)
    check_output(case, tensor_to_host(after), ids)
    assert v["counts"][8:].sum() > 0                     # the new slots are in use


def test_fill_of_a_live_slot_and_same_stream_are_rejected():
    import torch
    from gpu_util import Case
    from paper_2510_02613_amd import binding as B
    wl = MoEWorkload(name="fill_err", tokens=16, **MID)
    map_a, _ = relayout_maps(wl)
    case = Case(wl, expert_map=map_a)
    dev = case.x_dev.device
    copy = torch.cuda.Stream(device=dev)
    serve = torch.cuda.current_stream(dev)
    w13 = case.layer.upload(case.inp["w13_experts"][9])
    w2 = case.layer.upload(case.inp["w2_experts"][9])
    with pytest.raises(B.MoEError, match="active map"):
        case.layer.load_expert_async(3, w13, w2, copy, serve)           # slot 3 holds expert 3
    with pytest.raises(B.MoEError, match="differ"):
        case.layer.load_expert_async(12, w13, w2, serve, serve)
    with pytest.raises(B.MoEError, match="outside"):
        case.layer.load_expert_async(16, w13, w2, copy, serve)
    case.layer.load_expert_async(12, w13, w2, copy, serve)               # a free slot is fine
    torch.cuda.synchronize()
