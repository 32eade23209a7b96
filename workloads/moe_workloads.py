"""Synthetic stand-ins for the MoE layers of the models the paper serves.

The paper (Sec. 5, experimental setup) evaluates on trained DeepSeek-V2-Lite,
Qwen3-30B-A3B and DeepSeek-V3 checkpoints.  None of those weights exist here, so
each workload below only takes the *layer shape* of such a model (expert count
and top-k as the paper lists them; hidden / intermediate sizes from the public
model cards) and fills it with seeded random tensors:

  activations  N(0, 1)
  weights      N(0, 0.02)
  router       N(0, 0.02), or U(-0.02*sqrt(3), 0.02*sqrt(3)) ("uniform" router:
               same variance, expert load uniform in expectation)
  Zipf skew    logit_bias[e] = -s * ln(rank(e)), rank a random permutation of
               1..E, so that expert popularity falls off as rank**-s

Every tensor is drawn in fp32 from its own child of one SeedSequence and, for
bf16 workloads, rounded to nearest-even bf16; the rounded values are what both
the oracle and the GPU path consume.  bf16 tensors are carried as uint16 bit
patterns (`bf16_bits_to_f32` widens them exactly).

Nothing in this module computes any part of the MoE layer.
"""
from __future__ import annotations

import dataclasses
import math
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Optional, Tuple

import numpy as np

# ----------------------------------------------------------------------------
# bf16 <-> fp32 bit helpers (storage format conversion only)
# ----------------------------------------------------------------------------


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 -> bf16 (nearest, ties to even); returns uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    # no NaN/Inf appear in the synthetic draws, so the plain carry trick is exact
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to the fp32 values they denote (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# workload descriptions
# ----------------------------------------------------------------------------


@dataclasses.dataclass(frozen=True)
class MoEWorkload:
    name: str
    tokens: int  # T
    hidden: int  # H
    inter: int  # I   (SwiGLU intermediate of one expert)
    n_experts: int  # E   logical (global) routed experts
    top_k: int  # k
    n_slots: int  # S   physical weight slots on this rank (incl. shared)
    n_local: int  # logical experts [0, n_local) are the ones ever resident here
    act_dtype: str  # "f32" | "bf16"  (x, expert weights, out)
    router_dtype: str  # "f32" | "bf16"
    gate: str  # "softmax" | "sigmoid_group"
    n_group: int = 1
    topk_group: int = 1
    renormalize: bool = True
    routed_scale: float = 1.0
    n_shared: int = 0
    shared_range: Tuple[int, int] = (0, 0)  # tokens the shared expert serves
    router_dist: str = "normal"  # "normal" | "uniform"
    zipf_s: float = 0.0  # 0 = no skew
    seed: int = 0

    def with_tokens(self, tokens: int, shared_range=None) -> "MoEWorkload":
        sr = self.shared_range if shared_range is None else shared_range
        sr = (min(sr[0], tokens), min(sr[1], tokens))
        return dataclasses.replace(self, tokens=tokens, shared_range=sr)


WORKLOADS: Dict[str, MoEWorkload] = {
    # config 0: tiny fp32 layer, all experts local
    "tiny_f32": MoEWorkload(
        name="tiny_f32", tokens=64, hidden=128, inter=64, n_experts=8, top_k=2,
        n_slots=8, n_local=8, act_dtype="f32", router_dtype="f32", gate="softmax",
        seed=1),
    # config 1: Qwen3-30B-A3B-shaped layer, EP=1
    "qwen3_30b_a3b": MoEWorkload(
        name="qwen3_30b_a3b", tokens=4096, hidden=2048, inter=768, n_experts=128,
        top_k=8, n_slots=128, n_local=128, act_dtype="bf16", router_dtype="f32",
        gate="softmax", router_dist="uniform", seed=2),
    # config 2: DeepSeek-V3-shaped layer, one rank of EP=8 (32 routed + 1 shared)
    "dsv3_ep8_rank": MoEWorkload(
        name="dsv3_ep8_rank", tokens=8192, hidden=7168, inter=2048, n_experts=256,
        top_k=8, n_slots=33, n_local=32, act_dtype="bf16", router_dtype="bf16",
        gate="sigmoid_group", n_group=8, topk_group=4, routed_scale=2.5,
        n_shared=1, shared_range=(0, 1024), seed=3),
    # config 3: the same rank at decode batch size
    "dsv3_ep8_decode": MoEWorkload(
        name="dsv3_ep8_decode", tokens=64, hidden=7168, inter=2048, n_experts=256,
        top_k=8, n_slots=33, n_local=32, act_dtype="bf16", router_dtype="bf16",
        gate="sigmoid_group", n_group=8, topk_group=4, routed_scale=2.5,
        n_shared=1, shared_range=(0, 8), seed=4),
    # config 4: Qwen3 shape, Zipf-skewed routing, 32 -> 64 local experts in 64 slots
    "qwen3_relayout": MoEWorkload(
        name="qwen3_relayout", tokens=4096, hidden=2048, inter=768, n_experts=128,
        top_k=8, n_slots=64, n_local=64, act_dtype="bf16", router_dtype="f32",
        gate="softmax", zipf_s=1.2, seed=5),
    # beyond the five measured configs: the layer shape of the third model the paper serves
    # (Sec. 5), DeepSeek-V2-Lite-like: 64 routed experts, top-6 without renormalisation, 2 shared experts
    "dsv2_lite": MoEWorkload(
        name="dsv2_lite", tokens=4096, hidden=2048, inter=1408, n_experts=64,
        top_k=6, n_slots=66, n_local=64, act_dtype="bf16", router_dtype="f32",
        gate="softmax", renormalize=False, routed_scale=1.0,
        n_shared=2, shared_range=(0, 4096), seed=6),
}


def get_workload(name: str) -> MoEWorkload:
    return WORKLOADS[name]


# ----------------------------------------------------------------------------
# tensor generation
# ----------------------------------------------------------------------------

_TID = {"x": 0, "router": 1, "w13": 2, "w2": 3, "zipf_rank": 4, "slot_shuffle": 5}


def _rng(seed: int, tensor: str, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, _TID[tensor], sub])))


def _store(a: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return f32_to_bf16_bits(a)
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    raise ValueError(dtype)


def _normal(seed, tensor, sub, shape, std, dtype):
    a = _rng(seed, tensor, sub).standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return _store(a, dtype)


def make_inputs(wl: MoEWorkload, threads: int = 8) -> Dict[str, Optional[np.ndarray]]:
    """Draw every tensor of a workload.

    Returns a dict with
      x            [T, H]                 act dtype
      router_w     [E, H]                 router dtype
      logit_bias   [E] fp32 or None       (Zipf skew only)
      w13_experts  [n_local+n_shared, 2I, H]  per LOGICAL expert, rows 0..I-1 the
                   gate projection, I..2I-1 the up projection; shared experts last
      w2_experts   [n_local+n_shared, H, I]   down projection
    bf16 tensors are uint16 bit patterns, fp32 tensors are float32 arrays.
    """
    T, H, I, E = wl.tokens, wl.hidden, wl.inter, wl.n_experts
    n_w = wl.n_local + wl.n_shared
    out: Dict[str, Optional[np.ndarray]] = {}
    out["x"] = _normal(wl.seed, "x", 0, (T, H), 1.0, wl.act_dtype)
    if wl.router_dist == "uniform":
        a = 0.02 * math.sqrt(3.0)
        r = _rng(wl.seed, "router").random((E, H), dtype=np.float32)
        r = (r * np.float32(2 * a) - np.float32(a)).astype(np.float32)
        out["router_w"] = _store(r, wl.router_dtype)
    else:
        out["router_w"] = _normal(wl.seed, "router", 0, (E, H), 0.02, wl.router_dtype)
    if wl.zipf_s > 0.0:
        rank = _rng(wl.seed, "zipf_rank").permutation(E) + 1  # rank[e] in 1..E
        out["logit_bias"] = (-wl.zipf_s * np.log(rank.astype(np.float64))).astype(np.float32)
    else:
        out["logit_bias"] = None

    np_dt = np.uint16 if wl.act_dtype == "bf16" else np.float32
    w13 = np.empty((n_w, 2 * I, H), dtype=np_dt)
    w2 = np.empty((n_w, H, I), dtype=np_dt)

    def fill(e):
        w13[e] = _normal(wl.seed, "w13", e, (2 * I, H), 0.02, wl.act_dtype)
        w2[e] = _normal(wl.seed, "w2", e, (H, I), 0.02, wl.act_dtype)

    if n_w * I * H > (1 << 24) and threads > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(n_w)))
    else:
        for e in range(n_w):
            fill(e)
    out["w13_experts"] = w13
    out["w2_experts"] = w2
    return out


# ----------------------------------------------------------------------------
# expert placement (which logical expert lives in which physical slot)
# ----------------------------------------------------------------------------


def block_expert_map(n_experts: int, first: int, count: int, slots=None) -> np.ndarray:
    """Logical experts [first, first+count) are local; expert first+i -> slots[i]
    (default slot i).  Every other entry is -1 (not on this rank)."""
    m = np.full(n_experts, -1, dtype=np.int32)
    if slots is None:
        slots = np.arange(count, dtype=np.int32)
    m[first:first + count] = np.asarray(slots, dtype=np.int32)
    return m


def relayout_maps(wl: MoEWorkload) -> Tuple[np.ndarray, np.ndarray]:
    """The two placements of the re-layout workload.

    Phase A: logical experts 0..S/2-1 sit in slots of the same number, the other
    half of the pool is empty (EP=4 share of 128 experts in a 64-slot pool).
    Phase B: experts S/2..S-1 have been copied into the free slots in a shuffled
    order (EP=2 share); the first half has not moved.
    """
    half = wl.n_slots // 2
    a = block_expert_map(wl.n_experts, 0, half)
    shuffle = _rng(wl.seed, "slot_shuffle").permutation(half).astype(np.int32) + half
    b = a.copy()
    b[half:2 * half] = shuffle
    return a, b


def shared_slots_of(wl: MoEWorkload) -> np.ndarray:
    """Shared experts occupy the last n_shared slots of the pool."""
    return np.arange(wl.n_slots - wl.n_shared, wl.n_slots, dtype=np.int32)


def build_slot_pool(experts: np.ndarray, expert_map: np.ndarray, n_slots: int,
                    n_local: int, shared_slots=(), fill=None) -> np.ndarray:
    """Lay per-logical-expert weights out as the physical slot pool [S, ...].

    pool[expert_map[e]] = experts[e] for every local e; pool[shared_slots[i]] =
    experts[n_local + i].  Slots nothing maps to are filled with `fill`
    (default: NaN, so that a kernel reading a dead slot is caught).
    """
    pool = np.empty((n_slots,) + experts.shape[1:], dtype=experts.dtype)
    if fill is None:
        fill = np.uint16(0x7FC0) if experts.dtype == np.uint16 else np.float32("nan")
    pool[...] = fill
    for e, s in enumerate(np.asarray(expert_map)):
        if s >= 0:
            if e >= n_local:
                raise ValueError(f"expert {e} mapped to a slot but has no weights here")
            pool[s] = experts[e]
    for i, s in enumerate(shared_slots):
        pool[s] = experts[n_local + i]
    return pool
