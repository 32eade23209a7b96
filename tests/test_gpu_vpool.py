"""The weight pools as contiguous virtual tensors over physical pages (moe_vpool_*): growth by mapping
fresh pages behind the resident ones, re-placement of experts by exchanging pages (no byte moves),
shrink -- each checked against the oracle or for bit-identical outputs."""
import numpy as np
import pytest

from workloads import MoEWorkload

pytestmark = pytest.mark.gpu

MID = dict(hidden=512, inter=264, n_experts=32, top_k=4, n_slots=16, n_local=16,
           act_dtype="bf16", router_dtype="f32", gate="softmax", seed=41)


def _check(case):
    from gpu_util import check_routing, check_bookkeeping, check_output
    wl = case.wl
    out = case.run()
    v = case.layer.view(wl.tokens)
    ids, _, _ = check_routing(case, v["topk_ids"], v["topk_w"])
    check_bookkeeping(case, v, wl.tokens, wl.shared_range)
    check_output(case, out, ids)
    return out


def test_virtual_pool_grow_replace_shrink():
    import torch
    from gpu_util import Case, tensor_to_host
    from paper_2510_02613_amd.layer import VirtualPool
    wl = MoEWorkload(name="vpool", tokens=900, **MID)
    H, I, S = wl.hidden, wl.inter, wl.n_slots
    p13 = VirtualPool(S, (2 * I, H), torch.int16)
    p2 = VirtualPool(S, (H, I), torch.int16)
    try:
        # 8 resident experts: pages allocated in one order, mapped under slots 0..7 in another
        pages13 = [p13.page_alloc() for _ in range(8)]
        pages2 = [p2.page_alloc() for _ in range(8)]
        for s in range(8):
            p13.map(s, pages13[7 - s])
            p2.map(s, pages2[(s + 3) % 8])
        map_a = np.full(wl.n_experts, -1, np.int32)
        map_a[:8] = np.arange(8)
        case = Case(wl, expert_map=map_a, pools=(p13, p2))
        assert case.layer.w13.data_ptr() == p13.tensor.data_ptr()
        out_a = _check(case)

        # grow: fresh pages mapped behind the resident ones, filled in the background, then the switch
        base = (p13.tensor.data_ptr(), p2.tensor.data_ptr())
        for s in range(8, 16):
            p13.map(s, p13.page_alloc())
            p2.map(s, p2.page_alloc())
        copy = torch.cuda.Stream()
        src = [(case.layer.upload(case.inp["w13_experts"][e]), case.layer.upload(case.inp["w2_experts"][e])) for e in range(8, 16)]
        for e in range(8, 16):
            case.layer.load_expert_async(e, src[e - 8][0], src[e - 8][1], copy)
        map_b = map_a.copy()
        map_b[8:16] = np.arange(8, 16)                 # contiguous: expert e in virtual slot e
        case.place(map_b, upload=False)
        assert base == (case.layer.w13.data_ptr(), case.layer.w2.data_ptr())
        out_b = _check(case)
        np.testing.assert_array_equal(tensor_to_host(p13.tensor[:16]), case.w13_pool)

        # re-place without moving a byte: exchange the pages under slots 3 and 12, and the map entries
        torch.cuda.synchronize()
        for pool in (p13, p2):
            a, b = pool.page_of(3), pool.page_of(12)
            pool.unmap(3)
            pool.unmap(12)
            pool.map(3, b)
            pool.map(12, a)
        np.testing.assert_array_equal(tensor_to_host(p13.tensor[3]), case.inp["w13_experts"][12])
        np.testing.assert_array_equal(tensor_to_host(p2.tensor[12]), case.inp["w2_experts"][3])
        map_c = map_b.copy()
        map_c[3], map_c[12] = 12, 3
        case.place(map_c, upload=False)
        out_c = _check(case)
        np.testing.assert_array_equal(out_c, out_b)     # same experts, same weights, same sums

        # shrink back to the first 8 experts: expert 3 now lives under slot 12, so it stays; slot 3 (expert 12) goes
        map_d = map_a.copy()
        map_d[3] = 12
        case.place(map_d, upload=False)
        out_d = case.run()
        np.testing.assert_array_equal(out_d, out_a)
        torch.cuda.synchronize()
        for s in [3, 8, 9, 10, 11, 13, 14, 15]:
            for pool in (p13, p2):
                page = pool.page_of(s)
                pool.unmap(s)
                pool.page_free(page)
        np.testing.assert_array_equal(case.run(), out_a)   # the remaining pages are untouched
        case.layer.close()
    finally:
        torch.cuda.synchronize()
        p13.close()
        p2.close()


def test_virtual_pool_bookkeeping_errors():
    import torch
    from paper_2510_02613_amd import binding as B
    from paper_2510_02613_amd.layer import VirtualPool
    with pytest.raises(B.MoEError) as ei:
        B.moe_vpool_create(4096 + 16, 4)               # slots could not lie back to back
    assert ei.value.status == B.MOE_ERR_UNSUPPORTED
    pool = VirtualPool(4, (64, 64), torch.float32)      # 16 KB slots
    try:
        a, b = pool.page_alloc(), pool.page_alloc()
        pool.map(0, a)
        assert pool.page_of(0) == a and pool.page_of(1) == -1
        for call in (lambda: pool.map(0, b),            # slot taken
                     lambda: pool.map(1, a),            # page taken
                     lambda: pool.page_free(a),         # still mapped
                     lambda: pool.unmap(2)):            # nothing there
            with pytest.raises(B.MoEError) as ei:
                call()
            assert ei.value.status == B.MOE_ERR_MAP
        with pytest.raises(B.MoEError):
            pool.map(4, b)
        pool.tensor[0].fill_(1.5)
        pool.unmap(0)
        pool.map(3, a)                                  # the page keeps its contents
        torch.cuda.synchronize()
        assert float(pool.tensor[3].min()) == 1.5 and float(pool.tensor[3].max()) == 1.5
        pool.page_free(b)
    finally:
        pool.close()


def test_bound_pools_refuse_slots_without_a_page():
    """A layer that knows its page pools turns what would be a GPU fault into MOE_ERR_MAP on the host: a
    placement naming a slot without a page, a fill into one, a forward after a page of the placement in
    force was taken away -- and runs as before once the page is back."""
    import torch
    from gpu_util import Case
    from paper_2510_02613_amd import binding as B
    from paper_2510_02613_amd.layer import VirtualPool
    wl = MoEWorkload(name="vpool_guard", tokens=300, **MID)
    H, I, S = wl.hidden, wl.inter, wl.n_slots
    p13 = VirtualPool(S, (2 * I, H), torch.int16)
    p2 = VirtualPool(S, (H, I), torch.int16)
    other = VirtualPool(S, (H, I), torch.int16)
    try:
        for s in range(8):
            p13.map(s, p13.page_alloc())
            p2.map(s, p2.page_alloc())
        p13.map(9, p13.page_alloc())                        # slot 9: a page in the w13 pool only
        map_a = np.full(wl.n_experts, -1, np.int32)
        map_a[:8] = np.arange(8)
        case = Case(wl, expert_map=map_a, pools=(p13, p2))
        layer = case.layer
        out_a = _check(case)

        bad = map_a.copy()
        bad[8] = 9
        with pytest.raises(B.MoEError) as ei:
            layer.set_expert_map(bad)
        assert ei.value.status == B.MOE_ERR_MAP and "w2 pool" in str(ei.value)
        bad[8] = 10
        with pytest.raises(B.MoEError) as ei:
            layer.set_expert_map(bad)
        assert ei.value.status == B.MOE_ERR_MAP and "w13 pool" in str(ei.value)
        with pytest.raises(B.MoEError) as ei:
            layer.set_expert_replicas([[e, 10] if e == 0 else ([e] if e < 8 else []) for e in range(wl.n_experts)])
        assert ei.value.status == B.MOE_ERR_MAP
        np.testing.assert_array_equal(case.run(), out_a)    # the placement in force is untouched

        src = (layer.upload(case.inp["w13_experts"][8]), layer.upload(case.inp["w2_experts"][8]))
        with pytest.raises(B.MoEError) as ei:
            layer.load_expert_async(9, src[0], src[1], torch.cuda.Stream())
        assert ei.value.status == B.MOE_ERR_MAP

        torch.cuda.synchronize()                            # nothing in flight: a page of the active placement goes
        page = p13.page_of(5)
        p13.unmap(5)
        with pytest.raises(B.MoEError) as ei:
            case.run()
        assert ei.value.status == B.MOE_ERR_MAP and "slot 5" in str(ei.value)
        p13.map(5, page)                                    # the page kept its contents
        np.testing.assert_array_equal(case.run(), out_a)

        # binding checks: a pool that is not the layer's, and a placement in force that is not readable
        with pytest.raises(B.MoEError) as ei:
            B.moe_layer_bind_vpools(layer.handle, p13.handle, other.handle)
        assert ei.value.status == B.MOE_ERR_ARG
        with pytest.raises(B.MoEError) as ei:
            B.moe_layer_bind_vpools(layer.handle, p2.handle, None)     # wrong slot size and base
        assert ei.value.status == B.MOE_ERR_ARG
        B.moe_layer_bind_vpools(layer.handle, None, None)   # unbound: the host no longer looks
        p2.unmap(7)
        page7 = p2.page_of(7)
        assert page7 == -1
        with pytest.raises(B.MoEError) as ei:
            B.moe_layer_bind_vpools(layer.handle, p13.handle, p2.handle)
        assert ei.value.status == B.MOE_ERR_MAP and "slot 7" in str(ei.value)
        torch.cuda.synchronize()
        # a pool that goes away before the layer takes its checks with it
        B.moe_layer_bind_vpools(layer.handle, p13.handle, None)
    finally:
        torch.cuda.synchronize()
        p13.close()
        p2.close()
        other.close()
    case.layer.close()
