"""ctypes front end of the fp64 CPU oracle (oracle/moe_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the CPU
baseline leg of the benchmark.  The product package never imports this module
and this module never imports the product package.

The wrapper only marshals arrays; every step of the layer is in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")

F32, BF16 = 0, 1
GATE_SOFTMAX, GATE_SIGMOID_GROUP = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over tokens)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Cfg(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("H", ctypes.c_int32), ("I", ctypes.c_int32),
                ("E", ctypes.c_int32), ("k", ctypes.c_int32), ("S", ctypes.c_int32),
                ("gate", ctypes.c_int32), ("n_group", ctypes.c_int32),
                ("topk_group", ctypes.c_int32), ("renormalize", ctypes.c_int32),
                ("routed_scale", ctypes.c_double), ("n_shared", ctypes.c_int32),
                ("act_dtype", ctypes.c_int32), ("router_dtype", ctypes.c_int32)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_route.restype = None
        _lib.oracle_forward.restype = None
        _lib.oracle_forward_routed.restype = None
        _lib.oracle_forward_replicated.restype = None
        _lib.oracle_max_threads.restype = ctypes.c_int
    return _lib


def max_threads() -> int:
    return int(_load().oracle_max_threads())


@dataclass
class LayerSpec:
    """Shape and gating rule of the layer (mirrors the C struct)."""
    T: int
    H: int
    I: int
    E: int
    k: int
    S: int
    gate: str = "softmax"  # "softmax" | "sigmoid_group"
    n_group: int = 1
    topk_group: int = 1
    renormalize: bool = True
    routed_scale: float = 1.0
    n_shared: int = 0

    @staticmethod
    def from_workload(wl) -> "LayerSpec":
        return LayerSpec(T=wl.tokens, H=wl.hidden, I=wl.inter, E=wl.n_experts, k=wl.top_k,
                         S=wl.n_slots, gate=wl.gate, n_group=wl.n_group,
                         topk_group=wl.topk_group, renormalize=wl.renormalize,
                         routed_scale=wl.routed_scale, n_shared=wl.n_shared)


def _storage(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"oracle inputs are float32 arrays or uint16 bf16 bit patterns, got {a.dtype}")


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype=None):
    if a is None:
        return None
    a = np.ascontiguousarray(a) if dtype is None else np.ascontiguousarray(a, dtype=dtype)
    return a


def _cfg(spec: LayerSpec, x, router_w, w13=None) -> _Cfg:
    act = _storage(x)
    if w13 is not None and _storage(w13) != act:
        raise TypeError("x and expert weights must use the same storage type")
    assert x.shape == (spec.T, spec.H), (x.shape, spec)
    assert router_w is None or router_w.shape == (spec.E, spec.H)
    assert spec.E % max(spec.n_group, 1) == 0 and spec.n_group <= 256
    assert 1 <= spec.k <= spec.E
    return _Cfg(spec.T, spec.H, spec.I, spec.E, spec.k, spec.S,
                GATE_SOFTMAX if spec.gate == "softmax" else GATE_SIGMOID_GROUP,
                spec.n_group, spec.topk_group, int(spec.renormalize), float(spec.routed_scale),
                spec.n_shared, act, act if router_w is None else _storage(router_w))


def route(spec: LayerSpec, x, router_w, logit_bias=None, select_bias=None, want_scores=False):
    """Gate every token: returns (ids [T,k] int32, w [T,k] fp64, flags [T] uint8
    [, selection scores [T,E] fp32]).  flags bit0: expert near-tie, bit1: group near-tie."""
    x, router_w = _c(x), _c(router_w)
    logit_bias, select_bias = _c(logit_bias, np.float32), _c(select_bias, np.float32)
    cfg = _cfg(spec, x, router_w)
    ids = np.empty((spec.T, spec.k), dtype=np.int32)
    w = np.empty((spec.T, spec.k), dtype=np.float64)
    flags = np.zeros(spec.T, dtype=np.uint8)
    c = np.empty((spec.T, spec.E), dtype=np.float32) if want_scores else None
    _load().oracle_route(ctypes.byref(cfg), _ptr(x), _ptr(router_w), _ptr(logit_bias),
                         _ptr(select_bias), _ptr(ids), _ptr(w), _ptr(flags), _ptr(c))
    return (ids, w, flags, c) if want_scores else (ids, w, flags)


def forward(spec: LayerSpec, x, router_w, w13, w2, expert_map, *, logit_bias=None,
            select_bias=None, shared_slots: Sequence[int] = (), shared_range=(0, 0),
            tokens=None, forced_ids=None, identity_experts=False) -> np.ndarray:
    """Layer output rows (fp64) for `tokens` (default: all T tokens, in order)."""
    x, router_w, w13, w2 = _c(x), _c(router_w), _c(w13), _c(w2)
    logit_bias, select_bias = _c(logit_bias, np.float32), _c(select_bias, np.float32)
    cfg = _cfg(spec, x, router_w, w13)
    assert w13.shape == (spec.S, 2 * spec.I, spec.H), w13.shape
    assert w2.shape == (spec.S, spec.H, spec.I), w2.shape
    expert_map = _c(expert_map, np.int32)
    assert expert_map.shape == (spec.E,)
    assert expert_map.max(initial=-1) < spec.S and expert_map.min(initial=0) >= -1
    shared = _c(np.asarray(list(shared_slots), dtype=np.int32))
    assert shared.shape == (spec.n_shared,)
    tok = np.arange(spec.T, dtype=np.int32) if tokens is None else _c(tokens, np.int32)
    assert tok.size == 0 or (tok.min() >= 0 and tok.max() < spec.T)
    forced = _c(forced_ids, np.int32)
    if forced is not None:
        assert forced.shape == (spec.T, spec.k)
        assert forced.min() >= 0 and forced.max() < spec.E
    out = np.empty((tok.size, spec.H), dtype=np.float64)
    _load().oracle_forward(ctypes.byref(cfg), _ptr(x), _ptr(router_w), _ptr(logit_bias),
                           _ptr(select_bias), _ptr(w13), _ptr(w2), _ptr(expert_map),
                           _ptr(shared), ctypes.c_int32(int(shared_range[0])),
                           ctypes.c_int32(int(shared_range[1])), _ptr(tok),
                           ctypes.c_int32(int(tok.size)), _ptr(forced),
                           ctypes.c_int32(int(identity_experts)), _ptr(out))
    return out


def forward_routed(spec: LayerSpec, x, w13, w2, expert_map, ids, wts, *, shared_slots: Sequence[int] = (),
                   shared_range=(0, 0), tokens=None, identity_experts=False) -> np.ndarray:
    """Layer output rows (fp64) when the routing is given: ids [T,k] int32 (ids outside [0,E)
    are padding), wts [T,k] fp32 used as they are."""
    x, w13, w2 = _c(x), _c(w13), _c(w2)
    cfg = _cfg(spec, x, None, w13)
    assert w13.shape == (spec.S, 2 * spec.I, spec.H), w13.shape
    assert w2.shape == (spec.S, spec.H, spec.I), w2.shape
    expert_map = _c(expert_map, np.int32)
    assert expert_map.shape == (spec.E,)
    assert expert_map.max(initial=-1) < spec.S and expert_map.min(initial=0) >= -1
    shared = _c(np.asarray(list(shared_slots), dtype=np.int32))
    assert shared.shape == (spec.n_shared,)
    ids, wts = _c(ids, np.int32), _c(wts, np.float32)
    assert ids.shape == (spec.T, spec.k) and wts.shape == (spec.T, spec.k)
    tok = np.arange(spec.T, dtype=np.int32) if tokens is None else _c(tokens, np.int32)
    assert tok.size == 0 or (tok.min() >= 0 and tok.max() < spec.T)
    out = np.empty((tok.size, spec.H), dtype=np.float64)
    _load().oracle_forward_routed(ctypes.byref(cfg), _ptr(x), _ptr(w13), _ptr(w2), _ptr(expert_map),
                                  _ptr(shared), ctypes.c_int32(int(shared_range[0])),
                                  ctypes.c_int32(int(shared_range[1])), _ptr(tok),
                                  ctypes.c_int32(int(tok.size)), _ptr(ids), _ptr(wts),
                                  ctypes.c_int32(int(identity_experts)), _ptr(out))
    return out


def forward_replicated(spec: LayerSpec, x, router_w, w13, w2, replicas, *, logit_bias=None,
                       select_bias=None, shared_slots: Sequence[int] = (), shared_range=(0, 0),
                       tokens=None, forced_ids=None, identity_experts=False) -> np.ndarray:
    """Layer output rows (fp64) under a replicated placement: replicas[e] is the list of slots
    that hold a copy of logical expert e (empty: the expert is on another rank); token t uses
    copy t mod len(replicas[e])."""
    x, router_w, w13, w2 = _c(x), _c(router_w), _c(w13), _c(w2)
    logit_bias, select_bias = _c(logit_bias, np.float32), _c(select_bias, np.float32)
    cfg = _cfg(spec, x, router_w, w13)
    assert w13.shape == (spec.S, 2 * spec.I, spec.H), w13.shape
    assert w2.shape == (spec.S, spec.H, spec.I), w2.shape
    assert len(replicas) == spec.E
    rep_off = np.zeros(spec.E + 1, dtype=np.int32)
    rep_off[1:] = np.cumsum([len(r) for r in replicas])
    rep_slots = _c(np.asarray([s for r in replicas for s in r], dtype=np.int32))
    assert rep_slots.size == 0 or (rep_slots.min() >= 0 and rep_slots.max() < spec.S)
    shared = _c(np.asarray(list(shared_slots), dtype=np.int32))
    assert shared.shape == (spec.n_shared,)
    tok = np.arange(spec.T, dtype=np.int32) if tokens is None else _c(tokens, np.int32)
    assert tok.size == 0 or (tok.min() >= 0 and tok.max() < spec.T)
    forced = _c(forced_ids, np.int32)
    if forced is not None:
        assert forced.shape == (spec.T, spec.k)
        assert forced.min() >= 0 and forced.max() < spec.E
    out = np.empty((tok.size, spec.H), dtype=np.float64)
    _load().oracle_forward_replicated(ctypes.byref(cfg), _ptr(x), _ptr(router_w), _ptr(logit_bias),
                                      _ptr(select_bias), _ptr(w13), _ptr(w2), _ptr(rep_off), _ptr(rep_slots),
                                      _ptr(shared), ctypes.c_int32(int(shared_range[0])),
                                      ctypes.c_int32(int(shared_range[1])), _ptr(tok),
                                      ctypes.c_int32(int(tok.size)), _ptr(forced),
                                      ctypes.c_int32(int(identity_experts)), _ptr(out))
    return out
