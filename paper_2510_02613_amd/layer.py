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


class MoELayer:
    """One layer over caller-visible torch buffers.

    w13 / w2 are the physical slot pools [S,2I,H] / [S,H,I]; fill or refill slots
    with `load_slot`, then switch placement with `set_expert_map`.
    """

    def __init__(self, *, hidden, inter, n_experts, top_k, n_slots, max_tokens, act_dtype="bf16",
                 router_dtype="f32", gate="softmax", n_group=1, topk_group=1, renormalize=True,
                 routed_scale=1.0, n_shared=0, router_w: np.ndarray, logit_bias=None,
                 select_bias=None, device="cuda:0"):
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
        self.w13 = torch.empty((n_slots, 2 * inter, hidden), dtype=self.elt, device=self.device)
        self.w2 = torch.empty((n_slots, hidden, inter), dtype=self.elt, device=self.device)
        ws_bytes = B.moe_workspace_bytes(self.cfg)
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=self.device)
        self.buf = B.MoEBuffers(self.router_w.data_ptr(),
                                0 if self.logit_bias is None else self.logit_bias.data_ptr(),
                                0 if self.select_bias is None else self.select_bias.data_ptr(),
                                self.w13.data_ptr(), self.w2.data_ptr(),
                                self.workspace.data_ptr(), ws_bytes)
        self.handle = B.moe_layer_create(self.cfg, self.buf)

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
        es = 2 if self.act_dtype == "bf16" else 4
        npdt = np.uint16 if self.act_dtype == "bf16" else np.float32
        out["h"] = grab(v.h, es * A * self.cfg.inter, npdt, (A, self.cfg.inter))
        out["y"] = grab(v.y, es * A * self.cfg.hidden, npdt, (A, self.cfg.hidden))
        return out
