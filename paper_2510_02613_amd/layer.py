"""Device-buffer holder around the C ABI.

torch is plumbing here: it allocates device memory, copies host arrays in and
out, and names the stream.  Nothing in this file computes any step of the layer.
"""
from __future__ import annotations

from typing import Optional, Sequence

import numpy as np
import torch

from . import binding as B


def _dev(a: np.ndarray, device) -> torch.Tensor:
    """Upload a host array unchanged (uint16 bf16 bit patterns stay bit patterns)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device)
    return torch.from_numpy(a).to(device)


class _DeviceSpan:
    """Names a span of device memory for torch.as_tensor (no copy, no ownership)."""

    def __init__(self, ptr: int, shape, typestr: str):
        self.__cuda_array_interface__ = {"shape": tuple(shape), "typestr": typestr, "data": (ptr, False), "version": 2}


class VirtualPool:
    """A weight pool as one contiguous virtual tensor [n_vslots, *slot_shape] over separately
    allocated physical pages (the library's moe_vpool_* calls).  `tensor` is a torch view of the
    whole virtual range: index it only at slots that have a page."""

    def __init__(self, n_vslots: int, slot_shape, elt: torch.dtype, device="cuda:0"):
        self.device = torch.device(device)
        self.n_vslots, self.slot_shape, self.elt = n_vslots, tuple(slot_shape), elt
        esize = torch.empty((), dtype=elt).element_size()
        self.slot_bytes = int(np.prod(self.slot_shape)) * esize
        with torch.cuda.device(self.device):
            self.handle = B.moe_vpool_create(self.slot_bytes, n_vslots)
        typestr = {torch.int16: "<i2", torch.float32: "<f4"}[elt]
        self.tensor = torch.as_tensor(_DeviceSpan(B.moe_vpool_base(self.handle), (n_vslots,) + self.slot_shape, typestr),
                                      device=self.device)

    def page_alloc(self) -> int:
        return B.moe_vpool_page_alloc(self.handle)

    def page_free(self, page: int) -> None:
        B.moe_vpool_page_free(self.handle, page)

    def map(self, vslot: int, page: int) -> None:
        B.moe_vpool_map(self.handle, vslot, page)

    def unmap(self, vslot: int) -> None:
        B.moe_vpool_unmap(self.handle, vslot)

    def page_of(self, vslot: int) -> int:
        return B.moe_vpool_page_of(self.handle, vslot)

    def close(self) -> None:
        if getattr(self, "handle", None) is not None:
            self.tensor = None
            B.moe_vpool_destroy(self.handle)
            self.handle = None


class AttachedPool:
    """A weight pool that lives in ANOTHER process's device memory, opened through its exported handle
    (moe_pool_open): `tensor` is a torch view [n_vslots, *slot_shape] of it, nothing is copied or owned."""

    def __init__(self, handle: bytes, offset: int, n_vslots: int, slot_shape, elt: torch.dtype, device="cuda:0"):
        self.device = torch.device(device)
        self.n_vslots, self.slot_shape, self.elt, self.offset = n_vslots, tuple(slot_shape), elt, offset
        with torch.cuda.device(self.device):
            self.ptr = B.moe_pool_open(handle, offset)
        typestr = {torch.int16: "<i2", torch.float32: "<f4"}[elt]
        self.tensor = torch.as_tensor(_DeviceSpan(self.ptr, (n_vslots,) + self.slot_shape, typestr), device=self.device)

    def close(self) -> None:
        if getattr(self, "ptr", None):
            self.tensor = None
            B.moe_pool_close(self.ptr, self.offset)
            self.ptr = None


def export_pool(t: torch.Tensor):
    """(handle bytes, offset) of a pool tensor of this process, for AttachedPool in another process."""
    assert t.is_contiguous() and t.is_cuda
    return B.moe_pool_export(t.data_ptr())


class MoELayer:
    """One layer over caller-visible torch buffers.

    w13 / w2 are the physical slot pools [S,2I,H] / [S,H,I]; fill or refill slots
    with `load_slot`, then switch placement with `set_expert_map`.
    """

    def __init__(self, *, hidden, inter, n_experts, top_k, n_slots, max_tokens, act_dtype="bf16",
                 router_dtype="f32", gate="softmax", n_group=1, topk_group=1, renormalize=True,
                 routed_scale=1.0, n_shared=0, router_w: np.ndarray, logit_bias=None,
                 select_bias=None, device="cuda:0", w13_pool: Optional[VirtualPool] = None,
                 w2_pool: Optional[VirtualPool] = None):
        self.device = torch.device(device)
        dt = {"f32": B.MOE_F32, "bf16": B.MOE_BF16}
        self.cfg = B.MoEConfig(hidden, inter, n_experts, top_k, n_slots, max_tokens, dt[act_dtype],
                               dt[router_dtype], B.MOE_GATE_SOFTMAX_TOPK if gate == "softmax"
                               else B.MOE_GATE_SIGMOID_GROUP_TOPK, n_group, topk_group,
                               int(renormalize), float(routed_scale), n_shared)
        self.act_dtype = act_dtype
        self.elt = torch.int16 if act_dtype == "bf16" else torch.float32
        self.router_w = _dev(router_w, self.device)
        self.logit_bias = None if logit_bias is None else _dev(np.asarray(logit_bias, np.float32), self.device)
        self.select_bias = None if select_bias is None else _dev(np.asarray(select_bias, np.float32), self.device)
        # the pools: plain allocations, or views of virtual pools the caller maps pages under
        if w13_pool is None:
            self.w13 = torch.empty((n_slots, 2 * inter, hidden), dtype=self.elt, device=self.device)
        else:
            assert w13_pool.n_vslots == n_slots and w13_pool.slot_shape == (2 * inter, hidden) and w13_pool.elt == self.elt
            self.w13 = w13_pool.tensor
        if w2_pool is None:
            self.w2 = torch.empty((n_slots, hidden, inter), dtype=self.elt, device=self.device)
        else:
            assert w2_pool.n_vslots == n_slots and w2_pool.slot_shape == (hidden, inter) and w2_pool.elt == self.elt
            self.w2 = w2_pool.tensor
        ws_bytes = B.moe_workspace_bytes(self.cfg)
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=self.device)
        self.buf = B.MoEBuffers(self.router_w.data_ptr(),
                                0 if self.logit_bias is None else self.logit_bias.data_ptr(),
                                0 if self.select_bias is None else self.select_bias.data_ptr(),
                                self.w13.data_ptr(), self.w2.data_ptr(),
                                self.workspace.data_ptr(), ws_bytes)
        self.handle = B.moe_layer_create(self.cfg, self.buf)
        vp = [p.handle if isinstance(p, VirtualPool) else None for p in (w13_pool, w2_pool)]
        if vp[0] is not None or vp[1] is not None:
            # page pools: the host then refuses placements, fills and forwards that would touch a slot without a page
            B.moe_layer_bind_vpools(self.handle, vp[0], vp[1])

    def close(self):
        if getattr(self, "handle", None) is not None:
            B.moe_layer_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- weights -------------------------------------------------------------
    def load_slot(self, slot: int, w13: np.ndarray, w2: np.ndarray) -> None:
        """Copy one expert's weights into a physical slot (the stand-in for the paper's
        p2p-copy of an expert into freshly provided pages)."""
        self.w13[slot].copy_(_dev(w13, self.device))
        self.w2[slot].copy_(_dev(w2, self.device))

    def load_pool(self, w13_pool: np.ndarray, w2_pool: np.ndarray) -> None:
        self.w13.copy_(_dev(w13_pool, self.device))
        self.w2.copy_(_dev(w2_pool, self.device))

    def load_expert_async(self, slot: int, w13: torch.Tensor, w2: torch.Tensor, copy_stream: torch.cuda.Stream,
                          serve_stream: Optional[torch.cuda.Stream] = None, copy_blocks: int = 0) -> None:
        """Background fill of a slot that the active map does not use, from device tensors, on copy_stream;
        the next set_expert_map waits for it."""
        assert w13.dtype == self.elt and w13.is_contiguous() and tuple(w13.shape) == tuple(self.w13.shape[1:])
        assert w2.dtype == self.elt and w2.is_contiguous() and tuple(w2.shape) == tuple(self.w2.shape[1:])
        s = torch.cuda.current_stream(self.device) if serve_stream is None else serve_stream
        B.moe_load_expert(self.handle, slot, w13.data_ptr(), w2.data_ptr(), copy_stream.cuda_stream, s.cuda_stream,
                          copy_blocks)

    # -- placement -----------------------------------------------------------
    def set_expert_map(self, expert_map: Sequence[int], shared_slots: Optional[Sequence[int]] = None,
                       stream: Optional[torch.cuda.Stream] = None) -> None:
        s = torch.cuda.current_stream(self.device) if stream is None else stream
        B.moe_set_expert_map(self.handle, list(expert_map),
                             None if shared_slots is None or len(shared_slots) == 0 else list(shared_slots), s.cuda_stream)
        self.plain_map = ([int(v) for v in expert_map], None if shared_slots is None or len(shared_slots) == 0 else [int(v) for v in shared_slots])

    def set_expert_replicas(self, replicas: Sequence[Sequence[int]], shared_slots: Optional[Sequence[int]] = None,
                            stream: Optional[torch.cuda.Stream] = None) -> None:
        """Placement with copies: replicas[e] lists the slots holding expert e (empty: on another rank)."""
        s = torch.cuda.current_stream(self.device) if stream is None else stream
        offs = [0]
        for r in replicas:
            offs.append(offs[-1] + len(r))
        B.moe_set_expert_replicas(self.handle, offs, [int(v) for r in replicas for v in r],
                                  None if shared_slots is None or len(shared_slots) == 0 else list(shared_slots), s.cuda_stream)

    # -- forward -------------------------------------------------------------
    def upload(self, x: np.ndarray) -> torch.Tensor:
        return _dev(x, self.device)

    def forward(self, x: torch.Tensor, out: Optional[torch.Tensor] = None, shared_range=(0, 0),
                flags: int = 0, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
        assert x.dtype == self.elt and x.is_contiguous() and x.shape[1] == self.cfg.hidden
        T = x.shape[0]
        if out is None:
            out = torch.empty_like(x)
        s = torch.cuda.current_stream(self.device) if stream is None else stream
        B.moe_forward(self.handle, x.data_ptr(), T, out.data_ptr(), int(shared_range[0]),
                      int(shared_range[1]), s.cuda_stream, flags)
        return out

    def forward_static(self, x: torch.Tensor, out: Optional[torch.Tensor] = None, shared_range=(0, 0),
                       flags: int = 0, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
        """The same pass through moe_forward_static: this layer's configuration, weight buffers and last plain
        placement, every intermediate in the library's own device array (this layer's workspace is not used)."""
        assert x.dtype == self.elt and x.is_contiguous() and x.shape[1] == self.cfg.hidden
        if out is None:
            out = torch.empty_like(x)
        s = torch.cuda.current_stream(self.device) if stream is None else stream
        buf = B.MoEBuffers(self.buf.router_w, self.buf.logit_bias, self.buf.select_bias, self.buf.w13, self.buf.w2, 0, 0)
        B.moe_forward_static(self.cfg, buf, self.plain_map[0], self.plain_map[1], x.data_ptr(), x.shape[0], out.data_ptr(),
                             int(shared_range[0]), int(shared_range[1]), s.cuda_stream, flags)
        return out

    def forward_routed(self, x: torch.Tensor, topk_ids: torch.Tensor, topk_w: torch.Tensor,
                       out: Optional[torch.Tensor] = None, shared_range=(0, 0), flags: int = 0,
                       stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
        """The pass with the routing given (device int32 ids [T,k], float32 weights [T,k]); no gate."""
        assert x.dtype == self.elt and x.is_contiguous() and x.shape[1] == self.cfg.hidden
        T = x.shape[0]
        assert topk_ids.dtype == torch.int32 and topk_ids.is_contiguous() and tuple(topk_ids.shape) == (T, self.cfg.top_k)
        assert topk_w.dtype == torch.float32 and topk_w.is_contiguous() and tuple(topk_w.shape) == (T, self.cfg.top_k)
        assert topk_ids.device == x.device and topk_w.device == x.device
        if out is None:
            out = torch.empty_like(x)
        s = torch.cuda.current_stream(self.device) if stream is None else stream
        B.moe_forward_routed(self.handle, x.data_ptr(), T, topk_ids.data_ptr(), topk_w.data_ptr(), out.data_ptr(),
                             int(shared_range[0]), int(shared_range[1]), s.cuda_stream, flags)
        return out

    # -- intermediates (tests) -------------------------------------------------
    def view(self, T: int) -> dict:
        """Host copies of the intermediates of the last forward over T tokens."""
        v = B.moe_workspace_view(self.handle)
        base = self.workspace.data_ptr()
        k, kk, S = self.cfg.top_k, self.cfg.top_k + self.cfg.n_shared, self.cfg.n_slots

        def grab(ptr, nbytes, np_dtype, shape):
            off = ptr - base
            raw = self.workspace[off:off + nbytes].cpu().numpy()
            return raw.view(np_dtype).reshape(shape).copy()

        torch.cuda.synchronize(self.device)
        out = {
            "topk_ids": grab(v.topk_ids, 4 * T * k, np.int32, (T, k)),
            "topk_w": grab(v.topk_w, 4 * T * k, np.float32, (T, k)),
            "counts": grab(v.counts, 4 * S, np.int32, (S,)),
            "offsets": grab(v.offsets, 4 * (S + 1), np.int32, (S + 1,)),
            "inv": grab(v.inv, 4 * T * kk, np.int32, (T, kk)),
            "active_map": grab(v.active_map, 4 * (self.cfg.n_experts + self.cfg.n_shared), np.int32,
                               (self.cfg.n_experts + self.cfg.n_shared,)),
        }
        A = int(out["offsets"][S])
        out["perm"] = grab(v.perm, 4 * A, np.int32, (A,))
        n_tiles = int(grab(v.n_tiles, 4, np.int32, (1,))[0])
        out["tiles"] = grab(v.tiles, 16 * n_tiles, np.int32, (n_tiles, 4))   # slot, first grouped row, rows, single-tile flag
        # unit lists of the large-tile kernels (meaningful after a pass that ran them)
        out["unit_hdr"], out["units"] = None, None
        if v.unit_hdr:
            hdr = grab(v.unit_hdr, 32, np.int32, (2, 4))
            out["unit_hdr"] = hdr
            cap = (v.units1 - v.units0) // 16
            out["units"] = [grab(ptr, 16 * int(min(max(hdr[w, 2], 0), cap)), np.int32, (-1, 4)) for w, ptr in ((0, v.units0), (1, v.units1))]
        es = 2 if self.act_dtype == "bf16" else 4
        npdt = np.uint16 if self.act_dtype == "bf16" else np.float32
        out["h"] = grab(v.h, es * A * self.cfg.inter, npdt, (A, self.cfg.inter))
        out["y"] = grab(v.y, es * A * self.cfg.hidden, npdt, (A, self.cfg.hidden))
        return out
