"""Seeded synthetic activation tensors for the five benchmark configurations.

This module serves both the GPU tests/benchmark and the CPU oracle's tests.  It holds input
generation only — random draws, the per-channel structure and the conversion of the drawn
float32 numbers to bfloat16 bit patterns — and none of the compression method's arithmetic.

The paper evaluates on activations of real LLMs running Wikitext2 (Experiments, "Optimal
Compression Scheme Search"); neither the models nor the dataset are available here, so tensors
with the structure the paper's Background describes (a Gaussian or heavy-tailed body, a spread
of per-channel magnitudes, and a few persistent outlier channels that are the same for every
token and rank) stand in for them.

Recipe, for configuration seed ``s`` and rank ``r``::

    chan_scale[h]   = exp(0.5 * N(0,1))                drawn once from PCG64(s)
    outlier_idx     = sorted sample without replacement, drawn next from the same stream
    outlier_mult[h] = constant or U(lo, hi) on outlier_idx, 1 elsewhere
    body_r[t,h]     = N(0,1) or Student-t(nu=3)        from PCG64(s*1000 + r + 1)
    x_r[t,h]        = bf16_rne(body_r[t,h] * chan_scale[h] * outlier_mult[h])
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    tp: int
    tokens: int
    hidden: int
    seed: int
    body: str = "normal"                    # "normal" | "student_t3"
    n_outlier: int = 0
    outlier_mult: Tuple[float, float] = (1.0, 1.0)   # (lo, hi); lo == hi means a constant
    # (ebits, mbits, block, scale_bits) tuples the configuration sweeps
    formats: Tuple[Tuple[int, int, int, int], ...] = ((2, 1, 32, 8),)
    requantize: bool = False


CONFIGS = {
    1: Workload("tiny_tp2_128x1024", tp=2, tokens=128, hidden=1024, seed=0,
                n_outlier=4, outlier_mult=(50.0, 50.0)),
    2: Workload("llama8b_tp4_2048x4096", tp=4, tokens=2048, hidden=4096, seed=1,
                n_outlier=20, outlier_mult=(20.0, 100.0)),
    3: Workload("llama70b_tp8_4096x8192", tp=8, tokens=4096, hidden=8192, seed=2,
                n_outlier=41, outlier_mult=(20.0, 100.0),
                formats=((2, 1, 32, 8), (2, 2, 32, 8), (3, 2, 32, 8))),
    4: Workload("batched_tp8_8192x8192", tp=8, tokens=8192, hidden=8192, seed=3,
                body="student_t3", n_outlier=41, outlier_mult=(20.0, 100.0),
                formats=((2, 1, 16, 8), (2, 1, 32, 8)), requantize=True),
    5: Workload("llama405b_tp8_8192x16384", tp=8, tokens=8192, hidden=16384, seed=4,
                n_outlier=82, outlier_mult=(100.0, 100.0),
                formats=((2, 2, 32, 8),), requantize=True),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 bfloat16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> the float32 with the same value."""
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def channel_profile(w: Workload):
    """(chan_scale[H] float32, outlier_idx, outlier_mult[H] float32) shared by all ranks."""
    rng = np.random.Generator(np.random.PCG64(w.seed))
    chan_scale = np.exp(0.5 * rng.standard_normal(w.hidden)).astype(np.float32)
    mult = np.ones(w.hidden, dtype=np.float32)
    idx = np.sort(rng.choice(w.hidden, size=w.n_outlier, replace=False)) if w.n_outlier else \
        np.zeros(0, dtype=np.int64)
    lo, hi = w.outlier_mult
    if w.n_outlier:
        mult[idx] = lo if lo == hi else rng.uniform(lo, hi, size=w.n_outlier).astype(np.float32)
    return chan_scale, idx, mult


def partial_bf16(w: Workload, rank: int, rows: Optional[slice] = None) -> np.ndarray:
    """Rank ``rank``'s partial activation tensor as uint16 bf16 bit patterns [tokens, hidden].

    ``rows`` restricts the result to a row slice; the full tensor is still drawn so the values
    do not depend on the slice."""
    chan_scale, _, mult = channel_profile(w)
    rng = np.random.Generator(np.random.PCG64(w.seed * 1000 + rank + 1))
    body = rng.standard_normal((w.tokens, w.hidden), dtype=np.float32)
    if w.body == "student_t3":
        chi = rng.chisquare(3.0, size=(w.tokens, w.hidden)).astype(np.float32)
        body /= np.sqrt(chi / np.float32(3.0))
    elif w.body != "normal":
        raise ValueError(w.body)
    body *= (chan_scale * mult)[None, :]
    if rows is not None:
        body = body[rows]
    return f32_to_bf16_bits(body)


def all_partials_bf16(w: Workload, workers: int = 8):
    """Every rank's partial, drawn in parallel threads (the draws are independent streams, so
    the result is the same as calling partial_bf16 rank by rank)."""
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=max(1, min(workers, w.tp))) as pool:
        return list(pool.map(lambda r: partial_bf16(w, r), range(w.tp)))


def small_like(w: Workload, tokens: int, hidden: int) -> Workload:
    """The same distribution at a reduced shape (for tests the oracle finishes in seconds)."""
    n_out = max(1, round(w.n_outlier * hidden / w.hidden)) if w.n_outlier else 0
    return Workload(f"{w.name}_as_{tokens}x{hidden}", w.tp, tokens, hidden, w.seed, w.body,
                    n_out, w.outlier_mult, w.formats, w.requantize)


def stress_bf16(seed: int, tokens: int, hidden: int) -> np.ndarray:
    """A tensor built to stress a quantizer rather than to look like activations: per-block
    exponent ranges anywhere in bfloat16's span (subnormals and the largest binade included),
    random signs, and a sprinkle of +-0, Inf and NaN.  uint16 bit patterns [tokens, hidden]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    n = tokens * hidden
    # a base exponent per group of 8 elements, a few bits of spread around it per element
    base = rng.integers(0, 255, size=(n + 7) // 8)
    spread = rng.integers(-6, 1, size=n)
    expo = np.clip(np.repeat(base, 8)[:n] + spread, 0, 254).astype(np.uint16)
    mant = rng.integers(0, 128, size=n).astype(np.uint16)
    sign = rng.integers(0, 2, size=n).astype(np.uint16)
    bits = (sign << np.uint16(15)) | (expo << np.uint16(7)) | mant
    special = rng.random(n)
    bits[special < 0.02] &= np.uint16(0x8000)                       # +-0
    bits[(special >= 0.02) & (special < 0.021)] = np.uint16(0x7F80)  # +Inf
    bits[(special >= 0.021) & (special < 0.022)] = np.uint16(0xFF80)  # -Inf
    bits[(special >= 0.022) & (special < 0.023)] = np.uint16(0x7FC1)  # NaN
    return bits.reshape(tokens, hidden)
