"""Seeded synthetic attention inputs shaped like LLM inference.

This module only draws random numbers, casts them to the storage dtype and
plants structure (dominant keys).  It holds none of the attention arithmetic
and imports neither the HIP binding nor the CPU oracle, so both sides can be
fed from it without sharing any of the method's code.

All tensors are CPU torch tensors, contiguous, laid out
q: [B, Hq, Lq, d]   k, v: [B, Hkv, Lk, d].
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np
import torch

BASE_SEED = 20250514

TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


@dataclasses.dataclass(frozen=True)
class Workload:
    """One attention problem: shapes, dtype, mask and the value recipe."""
    name: str
    B: int
    Hq: int
    Hkv: int
    Lq: int
    Lk: int
    d: int
    dtype: str            # "f32" | "f16" | "bf16"
    causal: bool
    qk_std: float = 1.0   # Q and K are N(0, qk_std^2); V is always N(0, 1)
    plant_frac: float = 0.0  # fraction of query rows that get a dominant key 8*q
    seed: int = BASE_SEED
    sink_gain: float = 0.0   # > 0: per (b, kv head) one early key is set to
                             # (sink_gain / g) * sum of the group's last-position queries

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d)

    def visible_pairs(self) -> int:
        """Number of (query, key) pairs the mask leaves visible, per (b, h)."""
        if not self.causal:
            return self.Lq * self.Lk
        off = self.Lk - self.Lq
        n = 0
        for i in range(self.Lq):
            n += min(max(i + off + 1, 0), self.Lk)
        return n

    def flops(self) -> int:
        """Algorithmic flop: 2d for the score + 2d for the blend per visible pair."""
        return 4 * self.d * self.B * self.Hq * self.visible_pairs()

    def bytes_io(self) -> int:
        """Algorithmic bytes: every element of Q, K, V read once, O written once."""
        es = 4 if self.dtype == "f32" else 2
        nq = self.B * self.Hq * self.Lq * self.d
        nk = self.B * self.Hkv * self.Lk * self.d
        return es * (2 * nq + 2 * nk)


# The five configurations, in order.  Index 0 is the one a CPU finishes in
# well under a second; index 1 is the headline prefill case; index 3 is the
# headline decode case.
CONFIGS = (
    Workload("c1_single_head_f32", 1, 1, 1, 128, 128, 64, "f32", False, seed=BASE_SEED + 1),
    Workload("c2_llama7b_causal_prefill_bf16", 4, 32, 32, 2048, 2048, 128, "bf16", True,
             seed=BASE_SEED + 2),
    Workload("c3_long_noncausal_prefill_bf16", 1, 32, 32, 16384, 16384, 128, "bf16", False,
             seed=BASE_SEED + 3),
    Workload("c4_gqa_decode_bf16", 64, 32, 8, 1, 8192, 128, "bf16", False, seed=BASE_SEED + 4),
    Workload("c5_stability_stress_f16", 2, 16, 16, 4096, 4096, 64, "f16", True,
             qk_std=4.0, plant_frac=0.05, seed=BASE_SEED + 5),
)


def _normal(rng: np.random.Generator, shape, std: float, dtype: torch.dtype) -> torch.Tensor:
    x = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return torch.from_numpy(x).to(dtype).contiguous()   # round-to-nearest-even cast


def make_qkv(w: Workload):
    """Draw Q, K, V (in that order) for a workload and plant dominant keys.

    Planting: per (b, h) a Bernoulli(plant_frac) choice of query rows; for
    each chosen row i (ascending) a key index j uniform in the causally
    visible range [0, min(i + Lk - Lq, Lk - 1)] gets K[j] = 8 * Q[i] (exact in
    the storage dtype; later writes to the same j win).  Requires Hq == Hkv.
    """
    rng = np.random.default_rng(w.seed)
    dt = TORCH_DTYPE[w.dtype]
    q = _normal(rng, (w.B, w.Hq, w.Lq, w.d), w.qk_std, dt)
    k = _normal(rng, (w.B, w.Hkv, w.Lk, w.d), w.qk_std, dt)
    v = _normal(rng, (w.B, w.Hkv, w.Lk, w.d), 1.0, dt)
    planted = []
    if w.plant_frac > 0.0:
        if w.Hq != w.Hkv:
            raise ValueError("planting dominant keys needs Hq == Hkv")
        off = w.Lk - w.Lq
        for b in range(w.B):
            for h in range(w.Hq):
                sel = np.nonzero(rng.random(w.Lq) < w.plant_frac)[0]
                for i in sel:
                    hi = min(int(i) + off, w.Lk - 1) if w.causal else w.Lk - 1
                    if hi < 0:
                        continue
                    j = int(rng.integers(0, hi + 1))
                    k[b, h, j, :] = (q[b, h, int(i), :].float() * 8.0).to(dt)
                    planted.append((b, h, int(i), j))
    if w.sink_gain > 0.0:
        plant_group_sinks(w, q, k)
    return q, k, v, planted


def plant_group_sinks(w: Workload, q: torch.Tensor, k: torch.Tensor):
    """Peaked-score decode inputs, shaped like the attention sink of LLM decoding: per
    (b, kv head) one key among the first max(1, Lk // 64) positions (drawn from a generator of
    its own, seed + 7919, so that Q, K, V are the draws of the same workload without sinks) is
    set to (sink_gain / g) * sum over the g query heads of the group of their last-position
    query, rounded to the storage type.  Its score is then about sink_gain * |q|^2 * scale / g
    for every head of the group, far above the other keys', and every key after it has a
    weight that is exactly zero in fp32.  Returns the positions [B, Hkv]."""
    rng = np.random.default_rng(w.seed + 7919)
    g = w.Hq // w.Hkv
    pos = rng.integers(0, max(1, w.Lk // 64), size=(w.B, w.Hkv))
    for b in range(w.B):
        for kvh in range(w.Hkv):
            grp = q[b, kvh * g:(kvh + 1) * g, w.Lq - 1, :].float().sum(dim=0)
            k[b, kvh, int(pos[b, kvh]), :] = (grp * (w.sink_gain / g)).to(k.dtype)
    return pos


# The decode configuration with peaked scores: same shape, Q and K four times as wide, and a
# dominant early key per kv group (plant_group_sinks): the workload the saturation skip of
# Sec. III-C is measured on.
PEAKED_DECODE = Workload("c4p_gqa_decode_peaked_bf16", 64, 32, 8, 1, 8192, 128, "bf16", False,
                         qk_std=4.0, seed=BASE_SEED + 14, sink_gain=8.0)


def small(name: str, B, Hq, Hkv, Lq, Lk, d, dtype, causal, seed, qk_std=1.0,
          plant_frac=0.0, sink_gain=0.0) -> Workload:
    """A parity-test sized workload with an explicit seed."""
    return Workload(name, B, Hq, Hkv, Lq, Lk, d, dtype, causal, qk_std, plant_frac, seed,
                    sink_gain)


def sample_rows(w: Workload, n: int, seed: int, must=()):
    """Pick n distinct (b, h, i) query rows: first/last rows, rows around
    multiples of 32/64/128/256 (tile edges of any plausible kernel) and a
    seeded uniform remainder, plus every row in `must`."""
    rng = np.random.default_rng(seed)
    rows = set(tuple(int(x) for x in r) for r in must)
    edge_i = {0, 1, w.Lq - 1, w.Lq - 2}
    for t in (32, 64, 128, 256):
        for m in (1, 2, w.Lq // t - 1, w.Lq // t):
            for dlt in (-1, 0):
                edge_i.add(m * t + dlt)
    edge_i = sorted(i for i in edge_i if 0 <= i < w.Lq)
    for i in edge_i:
        rows.add((int(rng.integers(0, w.B)), int(rng.integers(0, w.Hq)), i))
    total = w.B * w.Hq * w.Lq
    n = min(n, total)
    while len(rows) < n:
        rows.add((int(rng.integers(0, w.B)), int(rng.integers(0, w.Hq)),
                  int(rng.integers(0, w.Lq))))
    return np.array(sorted(rows), dtype=np.int32)
