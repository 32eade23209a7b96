"""Host-only checks of the C ABI: the library loads, exports every declared symbol, and its
argument / expert-map validation works with no GPU (nothing here launches compute)."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2510_02613_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def good_cfg(**kw):
    d = dict(hidden=128, inter=64, n_experts=8, top_k=2, n_slots=8, max_tokens=64, act_dtype=0,
             router_dtype=0, gate=0, n_group=1, topk_group=1, renormalize=1, routed_scale=1.0, n_shared=0)
    d.update(kw)
    return B.MoEConfig(*[d[f] for f, _ in B.MoEConfig._fields_])


def fake_buffers(cfg, ws_bytes=None):
    # create never touches device memory, so aligned dummy addresses are enough on the host
    n = B.moe_workspace_bytes(cfg) if ws_bytes is None else ws_bytes
    return B.MoEBuffers(0x10000, 0, 0, 0x20000, 0x30000, 0x40000, n)


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "elasticmoe.h")).read()
    declared = set(re.findall(r"\b(moe_[a-z_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    lib = B.lib()
    for name in declared:
        assert hasattr(lib, name), name


def test_config_struct_matches_header_field_order():
    hdr = open(os.path.join(ROOT, "include", "elasticmoe.h")).read()
    body = hdr[hdr.index("typedef struct {\n    int32_t hidden"):hdr.index("} moe_config_t;")]
    names = re.findall(r"(?:int32_t|float)\s+(\w+);", body)
    assert names == [f for f, _ in B.MoEConfig._fields_]


@pytest.mark.parametrize("kw,status", [
    (dict(top_k=9), B.MOE_ERR_SHAPE),
    (dict(hidden=0), B.MOE_ERR_SHAPE),
    (dict(gate=1, n_group=3), B.MOE_ERR_SHAPE),
    (dict(gate=0, n_group=2, topk_group=1), B.MOE_ERR_SHAPE),
    (dict(gate=1, n_group=4, topk_group=5), B.MOE_ERR_SHAPE),
    (dict(gate=1, n_group=4, topk_group=1, top_k=3), B.MOE_ERR_SHAPE),
    (dict(act_dtype=7), B.MOE_ERR_ARG),
    (dict(gate=5), B.MOE_ERR_ARG),
    (dict(hidden=132), B.MOE_ERR_UNSUPPORTED),
    (dict(n_experts=2048, n_slots=8), B.MOE_ERR_UNSUPPORTED),
    (dict(n_shared=5, n_slots=16), B.MOE_ERR_UNSUPPORTED),
])
def test_bad_configs_are_rejected(kw, status):
    cfg = good_cfg(**kw)
    assert B.lib().moe_workspace_bytes(ctypes.byref(cfg)) == 0
    h = ctypes.c_void_p()
    buf = B.MoEBuffers(0x10000, 0, 0, 0x20000, 0x30000, 0x40000, 1 << 30)
    assert B.lib().moe_layer_create(ctypes.byref(cfg), ctypes.byref(buf), ctypes.byref(h)) == status
    assert h.value is None and B.moe_last_error()


def test_create_checks_pointers_alignment_and_workspace_size():
    cfg = good_cfg()
    need = B.moe_workspace_bytes(cfg)
    assert need > 0 and need % 256 == 0
    for mutate, status in [(lambda b: setattr(b, "w13", 0), B.MOE_ERR_ARG),
                           (lambda b: setattr(b, "w2", 0x30008), B.MOE_ERR_ARG),
                           (lambda b: setattr(b, "workspace", 0x40010), B.MOE_ERR_ARG),
                           (lambda b: setattr(b, "workspace_bytes", need - 1), B.MOE_ERR_CAPACITY)]:
        buf = fake_buffers(cfg)
        mutate(buf)
        with pytest.raises(B.MoEError) as ei:
            B.moe_layer_create(cfg, buf)
        assert ei.value.status == status
    h = B.moe_layer_create(cfg, fake_buffers(cfg))
    B.moe_layer_destroy(h)
    B.moe_layer_destroy(None)


def test_workspace_grows_with_capacity():
    a = B.moe_workspace_bytes(good_cfg(max_tokens=64))
    b = B.moe_workspace_bytes(good_cfg(max_tokens=128))
    assert b > a


def test_expert_map_validation_is_all_or_nothing():
    cfg = good_cfg(n_slots=10, n_shared=1)
    h = B.moe_layer_create(cfg, fake_buffers(cfg))
    try:
        ok_map = [0, 1, 2, -1, 4, 5, -1, 7]
        bad = [
            (ok_map[:7], [9]),                     # wrong length
            ([0, 1, 2, -2, 4, 5, -1, 7], [9]),     # entry below -1
            ([0, 1, 2, 10, 4, 5, -1, 7], [9]),     # slot out of range
            ([0, 1, 2, 2, 4, 5, -1, 7], [9]),      # two experts on one slot
            (ok_map, [4]),                         # shared slot also used by a routed expert
            (ok_map, [-1]),                        # a shared expert must have a slot
            (ok_map, None),                        # shared slots missing
        ]
        for m, s in bad:
            with pytest.raises(B.MoEError) as ei:
                B.moe_set_expert_map(h, m, s)
            assert ei.value.status == B.MOE_ERR_MAP, (m, s)
        # no map was installed by any of the rejected calls
        with pytest.raises(B.MoEError) as ei:
            B.moe_forward(h, 0x50000, 4, 0x60000)
        assert ei.value.status == B.MOE_ERR_MAP
        # forward argument checks come before anything is launched
        with pytest.raises(B.MoEError) as ei:
            B.moe_forward(h, 0x50000, 65, 0x60000)
        assert ei.value.status == B.MOE_ERR_CAPACITY
        with pytest.raises(B.MoEError) as ei:
            B.moe_forward(h, 0x50000, -1, 0x60000)
        assert ei.value.status == B.MOE_ERR_ARG
    finally:
        B.moe_layer_destroy(h)


def test_routed_forward_and_slot_fill_argument_checks():
    """Everything these two entry points reject is rejected before anything is launched."""
    cfg = good_cfg()
    h = B.moe_layer_create(cfg, fake_buffers(cfg))
    try:
        with pytest.raises(B.MoEError) as ei:       # routing missing
            B.moe_forward_routed(h, 0x50000, 4, 0, 0x70000, 0x60000)
        assert ei.value.status == B.MOE_ERR_ARG
        with pytest.raises(B.MoEError) as ei:       # same capacity rule as the gated pass
            B.moe_forward_routed(h, 0x50000, 65, 0x70000, 0x80000, 0x60000)
        assert ei.value.status == B.MOE_ERR_CAPACITY
        with pytest.raises(B.MoEError) as ei:       # no map yet
            B.moe_forward_routed(h, 0x50000, 4, 0x70000, 0x80000, 0x60000)
        assert ei.value.status == B.MOE_ERR_MAP
        for args in [(-1, 0x90000, 0xa0000, 1, 2, 0),     # slot below range
                     (8, 0x90000, 0xa0000, 1, 2, 0),      # slot past the pool
                     (3, 0, 0xa0000, 1, 2, 0),            # source missing
                     (3, 0x90008, 0xa0000, 1, 2, 0),      # source not 16-byte aligned
                     (3, 0x90000, 0xa0000, 1, 1, 0),      # copy stream == serving stream
                     (3, 0x90000, 0xa0000, 1, 2, -5)]:    # negative throttle
            with pytest.raises(B.MoEError) as ei:
                B.moe_load_expert(h, *args)
            assert ei.value.status == B.MOE_ERR_ARG, args
    finally:
        B.moe_layer_destroy(h)


def test_replicated_placement_argument_checks():
    """A placement with copies is validated on the host before anything is uploaded."""
    cfg = good_cfg(n_slots=12, n_shared=1)
    h = B.moe_layer_create(cfg, fake_buffers(cfg))
    try:
        ok_off = [0, 1, 4, 4, 6, 7, 8, 8, 9]                # expert 1 has 3 copies, 3 has 2, 2 and 6 are remote
        ok_slots = [0, 1, 10, 11, 2, 3, 4, 5, 6]
        bad = [
            (ok_off[:8], ok_slots, [9]),                    # wrong number of experts
            ([1] + ok_off[1:], ok_slots, [9]),              # offsets do not start at 0
            ([0, 1, 4, 3, 6, 7, 8, 8, 9], ok_slots, [9]),   # decreasing offsets
            ([0, 1, 4, 4, 6, 7, 8, 8, 13], ok_slots + [7, 8, 9, 9], [9]),   # more copies than slots
            (ok_off, [0, 1, 10, 12, 2, 3, 4, 5, 6], [9]),   # slot past the pool
            (ok_off, [0, 1, 10, -1, 2, 3, 4, 5, 6], [9]),   # a copy must have a slot
            (ok_off, [0, 1, 10, 1, 2, 3, 4, 5, 6], [9]),    # one slot for two copies of an expert
            (ok_off, [0, 1, 10, 11, 2, 3, 0, 5, 6], [9]),   # one slot for copies of two experts
            (ok_off, ok_slots, [11]),                       # shared slot also holds a copy
            (ok_off, ok_slots, None),                       # shared slots missing
        ]
        for o, r, s_ in bad:
            with pytest.raises(B.MoEError) as ei:
                B.moe_set_expert_replicas(h, o, r, s_)
            assert ei.value.status == B.MOE_ERR_MAP, (o, r, s_)
        with pytest.raises(B.MoEError) as ei:               # nothing was installed
            B.moe_forward(h, 0x50000, 4, 0x60000)
        assert ei.value.status == B.MOE_ERR_MAP
    finally:
        B.moe_layer_destroy(h)


def test_valid_map_without_gpu_fails_cleanly_or_installs():
    import torch
    if torch.cuda.is_available():
        pytest.skip("covered by the GPU tests")
    cfg = good_cfg()
    h = B.moe_layer_create(cfg, fake_buffers(cfg))
    try:
        with pytest.raises(B.MoEError) as ei:
            B.moe_set_expert_map(h, list(range(8)))
        assert ei.value.status == B.MOE_ERR_HIP     # no device: the upload kernel cannot launch
        with pytest.raises(B.MoEError) as ei:       # ... and the layer still has no map
            B.moe_forward(h, 0x50000, 4, 0x60000)
        assert ei.value.status == B.MOE_ERR_MAP
    finally:
        B.moe_layer_destroy(h)


def test_workloads_are_seeded_and_reproducible():
    from workloads import get_workload, make_inputs
    wl = get_workload("tiny_f32")
    a, b = make_inputs(wl), make_inputs(wl)
    for k in a:
        if a[k] is not None:
            np.testing.assert_array_equal(a[k], b[k])
    assert a["x"].shape == (64, 128) and a["w13_experts"].shape == (8, 128, 128)
    assert abs(float(a["w2_experts"].std()) - 0.02) < 2e-3


def test_virtual_pool_argument_checks_and_no_gpu():
    with pytest.raises(B.MoEError) as ei:
        B.moe_vpool_create(0, 4)
    assert ei.value.status == B.MOE_ERR_ARG
    with pytest.raises(B.MoEError) as ei:
        B.moe_vpool_create(4096, 0)
    assert ei.value.status == B.MOE_ERR_ARG
    assert B.moe_vpool_base(None) == 0 and B.moe_vpool_page_of(None, 0) == -1
    B.moe_vpool_destroy(None)
    assert B.moe_vpool_slot_bytes(None) == 0 and B.moe_vpool_slots(None) == 0
    with pytest.raises(B.MoEError) as ei:
        B.moe_layer_bind_vpools(None, None, None)
    assert ei.value.status == B.MOE_ERR_ARG
    import torch
    if not torch.cuda.is_available():
        with pytest.raises(B.MoEError) as ei:      # no device: nothing to reserve addresses on
            B.moe_vpool_create(4096, 4)
        assert ei.value.status in (B.MOE_ERR_HIP, B.MOE_ERR_UNSUPPORTED)


def test_ceiling_argument_checks():
    """The measuring-stick calls reject bad arguments before anything is launched."""
    L = B.lib()
    import ctypes
    assert L.moe_ceiling_stream(None, ctypes.c_size_t(4096), None, None) == B.MOE_ERR_ARG
    buf = ctypes.c_void_p(1 << 20)
    for n_tiles, row_bytes in ((0, 4096), (4, 0), (4, 100), (4, 1 << 24)):
        assert L.moe_ceiling_tile_stream(buf, n_tiles, ctypes.c_size_t(row_bytes), 0, None) == B.MOE_ERR_ARG
    assert L.moe_ceiling_tile_stream(None, 4, ctypes.c_size_t(4096), 0, None) == B.MOE_ERR_ARG
    assert L.moe_ceiling_tile_stream(ctypes.c_void_p((1 << 20) + 8), 4, ctypes.c_size_t(4096), 0, None) == B.MOE_ERR_ARG


def test_pool_export_argument_checks():
    import ctypes
    L = B.lib()
    h = ctypes.create_string_buffer(B.MOE_IPC_HANDLE_BYTES)
    off = ctypes.c_size_t()
    assert L.moe_pool_export(None, h, ctypes.byref(off)) == B.MOE_ERR_ARG
    assert L.moe_pool_export(ctypes.c_void_p(4096), None, ctypes.byref(off)) == B.MOE_ERR_ARG
    p = ctypes.c_void_p()
    assert L.moe_pool_open(None, 0, ctypes.byref(p)) == B.MOE_ERR_ARG
    assert L.moe_pool_open(h, 0, None) == B.MOE_ERR_ARG
    assert L.moe_pool_close(None, 0) == B.MOE_ERR_ARG
