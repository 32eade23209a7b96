"""ctypes binding of libelasticmoe.so: the same entry points, argument
marshalling only.  Every step of the layer runs in the HIP kernels; this module
holds no arithmetic and has no fallback: if the library is missing or a call
fails it raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libelasticmoe.so")

MOE_OK, MOE_ERR_ARG, MOE_ERR_SHAPE, MOE_ERR_MAP, MOE_ERR_CAPACITY, MOE_ERR_UNSUPPORTED, MOE_ERR_HIP = range(7)
MOE_F32, MOE_BF16 = 0, 1
MOE_GATE_SOFTMAX_TOPK, MOE_GATE_SIGMOID_GROUP_TOPK = 0, 1
MOE_FLAG_IDENTITY_EXPERTS, MOE_FLAG_FORCE_GENERIC, MOE_FLAG_GATE_TILED, MOE_FLAG_PERMUTE_UNFUSED = 1, 2, 4, 8

STATUS_NAMES = {0: "MOE_OK", 1: "MOE_ERR_ARG", 2: "MOE_ERR_SHAPE", 3: "MOE_ERR_MAP",
                4: "MOE_ERR_CAPACITY", 5: "MOE_ERR_UNSUPPORTED", 6: "MOE_ERR_HIP"}

# every symbol include/elasticmoe.h declares
EXPORTS = ("moe_workspace_bytes", "moe_layer_create", "moe_set_expert_map", "moe_forward",
           "moe_workspace_view", "moe_layer_destroy", "moe_last_error", "moe_profile_enable",
           "moe_profile_read", "moe_ceiling_mfma", "moe_ceiling_stream", "moe_forward_routed",
           "moe_load_expert", "moe_set_expert_replicas", "moe_vpool_create", "moe_vpool_base", "moe_vpool_page_alloc", "moe_vpool_page_free",
           "moe_vpool_map", "moe_vpool_unmap", "moe_vpool_page_of", "moe_vpool_destroy", "moe_vpool_slot_bytes",
           "moe_vpool_slots", "moe_layer_bind_vpools", "moe_ceiling_tile_stream", "moe_profile_select", "moe_forward_static",
           "moe_pool_export", "moe_pool_open", "moe_pool_close")
MOE_IPC_HANDLE_BYTES = 64
MOE_STATIC_SCRATCH_BYTES = 32 << 20
MOE_N_PHASES = 5
PHASE_NAMES = ("gate", "permute", "gemm1", "gemm2", "combine")


class MoEConfig(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int32), ("inter", ctypes.c_int32), ("n_experts", ctypes.c_int32),
                ("top_k", ctypes.c_int32), ("n_slots", ctypes.c_int32), ("max_tokens", ctypes.c_int32),
                ("act_dtype", ctypes.c_int32), ("router_dtype", ctypes.c_int32), ("gate", ctypes.c_int32),
                ("n_group", ctypes.c_int32), ("topk_group", ctypes.c_int32), ("renormalize", ctypes.c_int32),
                ("routed_scale", ctypes.c_float), ("n_shared", ctypes.c_int32)]


class MoEBuffers(ctypes.Structure):
    _fields_ = [("router_w", ctypes.c_void_p), ("logit_bias", ctypes.c_void_p),
                ("select_bias", ctypes.c_void_p), ("w13", ctypes.c_void_p), ("w2", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t)]


class MoEWorkspaceView(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("topk_ids", "topk_w", "counts", "offsets", "perm", "inv", "h", "y", "active_map", "tiles", "n_tiles",
                 "unit_hdr", "units0", "units1")]


class MoEError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status
        self.message = message


_lib = None


def lib() -> ctypes.CDLL:
    """Load libelasticmoe.so (built in-tree by paper_2510_02613_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2510_02613_amd.build` "
                              "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        L.moe_workspace_bytes.restype = ctypes.c_size_t
        L.moe_workspace_bytes.argtypes = [ctypes.POINTER(MoEConfig)]
        L.moe_layer_create.restype = ctypes.c_int
        L.moe_layer_create.argtypes = [ctypes.POINTER(MoEConfig), ctypes.POINTER(MoEBuffers),
                                       ctypes.POINTER(ctypes.c_void_p)]
        L.moe_set_expert_map.restype = ctypes.c_int
        L.moe_set_expert_map.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.c_int32,
                                         ctypes.POINTER(ctypes.c_int32), ctypes.c_void_p]
        L.moe_set_expert_replicas.restype = ctypes.c_int
        L.moe_set_expert_replicas.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32),
                                              ctypes.c_int32, ctypes.POINTER(ctypes.c_int32), ctypes.c_void_p]
        L.moe_forward.restype = ctypes.c_int
        L.moe_forward.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                  ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint32]
        L.moe_forward_routed.restype = ctypes.c_int
        L.moe_forward_routed.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_uint32]
        L.moe_forward_static.restype = ctypes.c_int
        L.moe_forward_static.argtypes = [ctypes.POINTER(MoEConfig), ctypes.POINTER(MoEBuffers), ctypes.POINTER(ctypes.c_int32),
                                         ctypes.c_int32, ctypes.POINTER(ctypes.c_int32), ctypes.c_void_p, ctypes.c_int32,
                                         ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint32]
        L.moe_load_expert.restype = ctypes.c_int
        L.moe_load_expert.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32]
        L.moe_vpool_create.restype = ctypes.c_int
        L.moe_vpool_create.argtypes = [ctypes.c_size_t, ctypes.c_int32, ctypes.POINTER(ctypes.c_void_p)]
        L.moe_vpool_base.restype = ctypes.c_void_p
        L.moe_vpool_base.argtypes = [ctypes.c_void_p]
        L.moe_vpool_page_alloc.restype = ctypes.c_int
        L.moe_vpool_page_alloc.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)]
        for name in ("moe_vpool_page_free", "moe_vpool_unmap"):
            getattr(L, name).restype = ctypes.c_int
            getattr(L, name).argtypes = [ctypes.c_void_p, ctypes.c_int32]
        L.moe_vpool_map.restype = ctypes.c_int
        L.moe_vpool_map.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32]
        L.moe_vpool_page_of.restype = ctypes.c_int32
        L.moe_vpool_page_of.argtypes = [ctypes.c_void_p, ctypes.c_int32]
        L.moe_vpool_destroy.restype = ctypes.c_int
        L.moe_vpool_destroy.argtypes = [ctypes.c_void_p]
        L.moe_vpool_slot_bytes.restype = ctypes.c_size_t
        L.moe_vpool_slot_bytes.argtypes = [ctypes.c_void_p]
        L.moe_vpool_slots.restype = ctypes.c_int32
        L.moe_vpool_slots.argtypes = [ctypes.c_void_p]
        L.moe_layer_bind_vpools.restype = ctypes.c_int
        L.moe_layer_bind_vpools.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.moe_pool_export.restype = ctypes.c_int
        L.moe_pool_export.argtypes = [ctypes.c_void_p, ctypes.c_char_p, ctypes.POINTER(ctypes.c_size_t)]
        L.moe_pool_open.restype = ctypes.c_int
        L.moe_pool_open.argtypes = [ctypes.c_char_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_void_p)]
        L.moe_pool_close.restype = ctypes.c_int
        L.moe_pool_close.argtypes = [ctypes.c_void_p, ctypes.c_size_t]
        L.moe_workspace_view.restype = ctypes.c_int
        L.moe_workspace_view.argtypes = [ctypes.c_void_p, ctypes.POINTER(MoEWorkspaceView)]
        L.moe_layer_destroy.restype = None
        L.moe_layer_destroy.argtypes = [ctypes.c_void_p]
        L.moe_profile_enable.restype = ctypes.c_int
        L.moe_profile_enable.argtypes = [ctypes.c_void_p, ctypes.c_int32]
        L.moe_profile_select.restype = ctypes.c_int
        L.moe_profile_select.argtypes = [ctypes.c_void_p, ctypes.c_int32]
        L.moe_profile_read.restype = ctypes.c_int
        L.moe_profile_read.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_float)]
        L.moe_ceiling_mfma.restype = ctypes.c_int
        L.moe_ceiling_mfma.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.POINTER(ctypes.c_double)]
        L.moe_ceiling_stream.restype = ctypes.c_int
        L.moe_ceiling_stream.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
        L.moe_ceiling_tile_stream.restype = ctypes.c_int
        L.moe_ceiling_tile_stream.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t, ctypes.c_int32, ctypes.c_void_p]
        L.moe_last_error.restype = ctypes.c_char_p
        L.moe_last_error.argtypes = []
        _lib = L
    return _lib


def moe_last_error() -> str:
    return lib().moe_last_error().decode()


def _check(status: int) -> None:
    if status != MOE_OK:
        raise MoEError(status, moe_last_error())


def moe_workspace_bytes(cfg: MoEConfig) -> int:
    n = lib().moe_workspace_bytes(ctypes.byref(cfg))
    if n == 0:
        raise MoEError(MOE_ERR_SHAPE, moe_last_error())
    return int(n)


def moe_layer_create(cfg: MoEConfig, buf: MoEBuffers) -> ctypes.c_void_p:
    h = ctypes.c_void_p()
    _check(lib().moe_layer_create(ctypes.byref(cfg), ctypes.byref(buf), ctypes.byref(h)))
    return h


def _i32_array(vals: Optional[Sequence[int]]):
    if vals is None:
        return None, 0
    vals = [int(v) for v in vals]
    return (ctypes.c_int32 * len(vals))(*vals), len(vals)


def moe_set_expert_map(layer, host_map: Sequence[int], host_shared_slots: Optional[Sequence[int]] = None,
                       stream: int = 0) -> None:
    m, n = _i32_array(host_map)
    s, ns = _i32_array(host_shared_slots)
    if ns == 0:
        s = None
    _check(lib().moe_set_expert_map(layer, m, n, s, ctypes.c_void_p(stream)))


def moe_set_expert_replicas(layer, host_rep_offsets: Sequence[int], host_rep_slots: Sequence[int],
                            host_shared_slots: Optional[Sequence[int]] = None, stream: int = 0) -> None:
    o, no = _i32_array(host_rep_offsets)
    r, nr = _i32_array(host_rep_slots)
    s, ns = _i32_array(host_shared_slots)
    _check(lib().moe_set_expert_replicas(layer, o, r if nr else None, no - 1, s if ns else None, ctypes.c_void_p(stream)))


def moe_forward(layer, x_ptr: int, T: int, out_ptr: int, shared_begin: int = 0, shared_end: int = 0,
                stream: int = 0, flags: int = 0) -> None:
    _check(lib().moe_forward(layer, ctypes.c_void_p(x_ptr), T, shared_begin, shared_end,
                             ctypes.c_void_p(out_ptr), ctypes.c_void_p(stream), flags))


def moe_forward_routed(layer, x_ptr: int, T: int, ids_ptr: int, w_ptr: int, out_ptr: int,
                       shared_begin: int = 0, shared_end: int = 0, stream: int = 0, flags: int = 0) -> None:
    _check(lib().moe_forward_routed(layer, ctypes.c_void_p(x_ptr), T, ctypes.c_void_p(ids_ptr), ctypes.c_void_p(w_ptr),
                                    shared_begin, shared_end, ctypes.c_void_p(out_ptr), ctypes.c_void_p(stream), flags))


def moe_forward_static(cfg: MoEConfig, buf: MoEBuffers, host_map: Sequence[int], host_shared_slots: Optional[Sequence[int]],
                       x_ptr: int, T: int, out_ptr: int, shared_begin: int = 0, shared_end: int = 0,
                       stream: int = 0, flags: int = 0) -> None:
    m, n = _i32_array(host_map)
    s, ns = _i32_array(host_shared_slots)
    _check(lib().moe_forward_static(ctypes.byref(cfg), ctypes.byref(buf), m, n, s if ns else None, ctypes.c_void_p(x_ptr), T,
                                    shared_begin, shared_end, ctypes.c_void_p(out_ptr), ctypes.c_void_p(stream), flags))


def moe_load_expert(layer, slot: int, src_w13_ptr: int, src_w2_ptr: int, copy_stream: int, serve_stream: int,
                    copy_blocks: int = 0) -> None:
    _check(lib().moe_load_expert(layer, slot, ctypes.c_void_p(src_w13_ptr), ctypes.c_void_p(src_w2_ptr),
                                 ctypes.c_void_p(copy_stream), ctypes.c_void_p(serve_stream), copy_blocks))


def moe_vpool_create(slot_bytes: int, n_vslots: int):
    h = ctypes.c_void_p()
    _check(lib().moe_vpool_create(ctypes.c_size_t(slot_bytes), n_vslots, ctypes.byref(h)))
    return h


def moe_vpool_base(pool) -> int:
    return int(lib().moe_vpool_base(pool) or 0)


def moe_vpool_page_alloc(pool) -> int:
    page = ctypes.c_int32(-1)
    _check(lib().moe_vpool_page_alloc(pool, ctypes.byref(page)))
    return int(page.value)


def moe_vpool_page_free(pool, page: int) -> None:
    _check(lib().moe_vpool_page_free(pool, page))


def moe_vpool_map(pool, vslot: int, page: int) -> None:
    _check(lib().moe_vpool_map(pool, vslot, page))


def moe_vpool_unmap(pool, vslot: int) -> None:
    _check(lib().moe_vpool_unmap(pool, vslot))


def moe_vpool_page_of(pool, vslot: int) -> int:
    return int(lib().moe_vpool_page_of(pool, vslot))


def moe_vpool_destroy(pool) -> None:
    _check(lib().moe_vpool_destroy(pool))


def moe_vpool_slot_bytes(pool) -> int:
    return int(lib().moe_vpool_slot_bytes(pool))


def moe_vpool_slots(pool) -> int:
    return int(lib().moe_vpool_slots(pool))


def moe_layer_bind_vpools(layer, w13_pool, w2_pool) -> None:
    """Either pool may be None (that buffer is plain memory)."""
    _check(lib().moe_layer_bind_vpools(layer, w13_pool, w2_pool))


def moe_pool_export(dev_ptr: int):
    """(handle bytes, offset) that name dev_ptr for another process."""
    handle = ctypes.create_string_buffer(MOE_IPC_HANDLE_BYTES)
    off = ctypes.c_size_t()
    _check(lib().moe_pool_export(ctypes.c_void_p(dev_ptr), handle, ctypes.byref(off)))
    return handle.raw, int(off.value)


def moe_pool_open(handle: bytes, offset: int) -> int:
    assert len(handle) == MOE_IPC_HANDLE_BYTES
    p = ctypes.c_void_p()
    _check(lib().moe_pool_open(ctypes.create_string_buffer(handle, MOE_IPC_HANDLE_BYTES), ctypes.c_size_t(offset), ctypes.byref(p)))
    return int(p.value)


def moe_pool_close(dev_ptr: int, offset: int) -> None:
    _check(lib().moe_pool_close(ctypes.c_void_p(dev_ptr), ctypes.c_size_t(offset)))


def moe_workspace_view(layer) -> MoEWorkspaceView:
    v = MoEWorkspaceView()
    _check(lib().moe_workspace_view(layer, ctypes.byref(v)))
    return v


def moe_profile_enable(layer, enable: int) -> None:
    """0 = off, n > 0 = record the phase events of every n-th forward."""
    _check(lib().moe_profile_enable(layer, int(enable)))


def moe_profile_select(layer, phase: int) -> None:
    """Record only the two events around one phase (-1: all phases again)."""
    _check(lib().moe_profile_select(layer, int(phase)))


def moe_profile_read(layer, back: int = 0):
    ms = (ctypes.c_float * MOE_N_PHASES)()
    _check(lib().moe_profile_read(layer, back, ms))
    return [float(v) for v in ms]


def moe_ceiling_mfma(blocks: int, iters: int, random_operands: bool, sink_ptr: int, stream: int = 0) -> float:
    """Enqueue the register-only MFMA stream; returns the flops of the launch."""
    flops = ctypes.c_double()
    _check(lib().moe_ceiling_mfma(blocks, iters, int(bool(random_operands)), ctypes.c_void_p(sink_ptr),
                                  ctypes.c_void_p(stream), ctypes.byref(flops)))
    return flops.value


def moe_ceiling_stream(buf_ptr: int, nbytes: int, sink_ptr: int, stream: int = 0) -> None:
    """Enqueue one streaming read of nbytes of device memory."""
    _check(lib().moe_ceiling_stream(ctypes.c_void_p(buf_ptr), ctypes.c_size_t(nbytes), ctypes.c_void_p(sink_ptr), ctypes.c_void_p(stream)))


def moe_ceiling_tile_stream(buf_ptr: int, n_tiles: int, row_bytes: int, non_temporal: bool, stream: int = 0) -> None:
    """Enqueue one read of n_tiles tiles of 256 rows x row_bytes in the access shape of the large-tile kernels' weight loaders."""
    _check(lib().moe_ceiling_tile_stream(ctypes.c_void_p(buf_ptr), ctypes.c_int32(n_tiles), ctypes.c_size_t(row_bytes),
                                         ctypes.c_int32(int(non_temporal)), ctypes.c_void_p(stream)))


def moe_layer_destroy(layer) -> None:
    lib().moe_layer_destroy(layer)
