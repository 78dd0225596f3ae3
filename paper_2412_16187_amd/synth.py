"""Seeded synthetic inputs for the HashEvict hot path.

This module only draws random tensors.  It contains none of the method's
arithmetic (no hashing, scoring, eviction or attention) and is the one piece
shared by the GPU tests, the benchmark and the CPU oracle's tests, so that both
sides see exactly the same numbers.

Every (sequence, layer, KV head) triple is one independent *unit*.  A unit's
tensors are drawn from ``numpy.random.Generator(PCG64(SeedSequence([seed,
unit])))`` in a fixed order, so any subset of units can be regenerated without
touching the others:

  1. channel scale ``s[d]``            LogNormal(0, sigma)   (all ones if sigma = 0)
  2. keys   ``K[N+T][d]``              s * N(0,1)
  3. values ``V[N+T][d]``              N(0,1)
  4. query source positions ``j[G][N+T]``  floor(U * t), U ~ Uniform[0,1)
  5. query noise ``E[G][N+T][d]``      N(0,1)
     ``Q[g][t] = mix * K[j[g][t]] + (1 - mix) * E[g][t]``   (mix = 0 -> Q = E)
  6. (needle workloads only) needle positions, directions and aligned queries.
  7. (``query_corr`` > 0 only) one common direction ``c[d] ~ N(0,1)`` per unit, drawn last so
     that the other tensors do not change: ``Q[g][t] += query_corr * |Q|_rms * sqrt(d) * c/|c|``
     -- every query of the unit shares a component of that relative weight, which makes the
     queries of consecutive tokens correlated as a real model's are (the benchmark
     configurations use 0).

The five named workloads follow the shapes and value distributions of the
benchmark configurations: Llama-3-8B-like attention geometry (32 layers, 32
query heads over 8 KV heads, head_dim 128), peaked attention produced by mixing
each query with an earlier key, and per-channel key scales.  They stand in for
the model activations the paper measured on; no dataset item or model weight is
used or needed.
"""
from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_layers: int
    n_kv_heads: int
    gqa_group: int
    head_dim: int
    hash_bits: int
    budget: int          # C, slots per unit
    n_prompt: int        # N
    n_decode: int        # T
    dtype: str           # "f32" or "bf16"
    seed: int
    key_scale_sigma: float = 0.5
    query_mix: float = 0.6
    needle_frac: float = 0.0
    needle_cos: float = 0.9
    n_sink: int = 0
    n_recent: int = 0
    policy: str = "hash"     # "hash" (HashEvict) or "l2" (the L2-norm comparator)
    query_corr: float = 0.0  # weight of a component shared by all queries of a unit (0 = independent)

    @property
    def n_units(self) -> int:
        return self.batch * self.n_layers * self.n_kv_heads

    @property
    def code_words(self) -> int:
        return (self.hash_bits + 31) // 32 if self.policy == "hash" else 1

    def scaled(self, **kw) -> "Workload":
        """Same recipe at other sizes (used by parity tests)."""
        return dataclasses.replace(self, **kw)


# The five benchmark configurations, in order.
TOY = Workload("toy", 1, 1, 4, 1, 128, 16, 256, 256, 512, "f32", 0,
               key_scale_sigma=0.0, query_mix=0.0)
LLAMA8B_DECODE = Workload("llama8b_decode", 1, 32, 8, 4, 128, 32, 2048, 4096, 256, "bf16", 1)
LLAMA8B_BATCH32 = Workload("llama8b_batch32", 32, 32, 8, 4, 128, 32, 1024, 2048, 128, "bf16", 2)
LONG_CONTEXT = Workload("long_context", 1, 1, 8, 4, 128, 32, 9830, 32768, 64, "bf16", 3,
                        needle_frac=0.01)
PREFILL = Workload("prefill", 8, 32, 8, 4, 128, 64, 2458, 8192, 0, "bf16", 4)

WORKLOADS = {w.name: w for w in (TOY, LLAMA8B_DECODE, LLAMA8B_BATCH32, LONG_CONTEXT, PREFILL)}


def unit_rng(seed: int, unit: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), int(unit)])))


def gen_unit(w: Workload, unit: int) -> dict:
    """Draw one unit's tensors as float32 arrays.

    Returns ``K``, ``V`` of shape ``[N+T][d]`` and ``Q`` of shape ``[G][N+T][d]``;
    rows ``< N`` are the prompt, rows ``>= N`` the decode steps in order.
    For needle workloads also ``needle_pos`` (sorted prompt positions).
    """
    d, G = w.head_dim, w.gqa_group
    n = w.n_prompt + w.n_decode
    rng = unit_rng(w.seed, unit)

    if w.key_scale_sigma > 0.0:
        s = np.exp(w.key_scale_sigma * rng.standard_normal(d, dtype=np.float32)).astype(np.float32)
    else:
        s = np.ones(d, dtype=np.float32)
    K = rng.standard_normal((n, d), dtype=np.float32) * s
    V = rng.standard_normal((n, d), dtype=np.float32)
    u = rng.random((G, n))
    t = np.arange(n, dtype=np.float64)
    j = np.floor(u * t).astype(np.int64)          # uniform over [0, t); 0 for t = 0
    E = rng.standard_normal((G, n, d), dtype=np.float32)
    out = {"scale": s}

    if w.needle_frac > 0.0:
        n_needle = max(1, int(round(w.needle_frac * w.n_prompt)))
        npos = np.sort(rng.choice(w.n_prompt, size=n_needle, replace=False))
        dirs = rng.standard_normal((n_needle, d)).astype(np.float64)
        dirs /= np.linalg.norm(dirs, axis=1, keepdims=True)
        knorm = float(np.linalg.norm(s))
        K[npos] = (knorm * dirs).astype(np.float32)
        out["needle_pos"] = npos

    if w.query_mix > 0.0:
        Q = np.float32(w.query_mix) * K[j] + np.float32(1.0 - w.query_mix) * E
    else:
        Q = E

    if w.needle_frac > 0.0:
        # Aligned queries: every decode query, and a needle_frac share of the
        # prompt queries that come after at least one needle.
        qnorm = math.sqrt(w.query_mix ** 2 * float(np.sum(s.astype(np.float64) ** 2))
                          + (1.0 - w.query_mix) ** 2 * d)
        pick = rng.random((G, n))
        which = rng.random((G, n))
        aligned = np.zeros((G, n), dtype=bool)
        aligned[:, w.n_prompt:] = True
        aligned[:, :w.n_prompt] = pick[:, :w.n_prompt] < w.needle_frac
        # number of needles strictly before position t
        n_before = np.searchsorted(npos, np.arange(n), side="left")
        aligned &= (n_before > 0)[None, :]
        gi, ti = np.nonzero(aligned)
        m = np.floor(which[gi, ti] * n_before[ti]).astype(np.int64)
        um = dirs[m]
        wv = E[gi, ti].astype(np.float64)
        wv -= np.sum(wv * um, axis=1, keepdims=True) * um
        wv /= np.linalg.norm(wv, axis=1, keepdims=True)
        c = w.needle_cos
        Q[gi, ti] = (qnorm * (c * um + math.sqrt(1.0 - c * c) * wv)).astype(np.float32)

    if w.query_corr > 0.0:
        c = rng.standard_normal(d)
        c /= np.linalg.norm(c)
        rms = float(np.sqrt(np.mean(np.square(Q, dtype=np.float64))))
        Q = Q + np.float32(w.query_corr * rms * math.sqrt(d)) * c.astype(np.float32)

    out.update(K=K, V=V, Q=np.ascontiguousarray(Q, dtype=np.float32))
    return out


def projection(w: Workload) -> np.ndarray:
    """The ``[d][r]`` N(0,1) projection matrix of a workload (float32)."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(w.seed), 0x5EED])))
    return rng.standard_normal((w.head_dim, w.hash_bits), dtype=np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + r) & np.uint32(0xFFFF0000)).view(np.float32)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of ``round_to_bf16(x)``."""
    return (round_to_bf16(x).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def quantize(w: Workload, x: np.ndarray) -> np.ndarray:
    """Values as both sides see them: bf16-rounded for bf16 workloads, else unchanged."""
    return round_to_bf16(x) if w.dtype == "bf16" else np.ascontiguousarray(x, dtype=np.float32)
