"""Seeded synthetic inputs for the split fully-connected + softmax head.

This module serves both the CPU oracle's tests and the HIP library's tests and
benchmark.  It holds none of the method's arithmetic: it only draws random
numbers, rounds them to bfloat16, and lists shard tables.  numpy only.

The workloads stand in for the paper's private 100K-class image data and its
ResNet50 pooled features (Section 1; Section 2.1; Section 5.1.2): same shapes
(D = 2048 features, C = 100 000 classes with a bias, which is what makes the
layer 782 MB in fp32), non-negative features, small-variance weights.

Conventions
  * RNG is numpy's Generator(PCG64(seed)); draw order is X, then W, then labels
    (then the bias, if one is asked for).
  * "N(0, s)" means standard deviation s.
  * Values are drawn in fp32, rounded once to bf16 (round to nearest even) and
    handed out as uint16 bit patterns; `bf16_bits_to_f64` upcasts them exactly,
    so the oracle and the GPU see identical numbers.
  * Zipf labels are a bounded Zipf: p_k proportional to (k + 1)^(-s), class id =
    rank k (hot classes first).
"""
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even) and return the 16-bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    is_nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    quiet = (u >> np.uint32(16)) | np.uint32(0x0040)
    return np.where(is_nan, quiet, rounded).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact upcast of bf16 bit patterns to float64."""
    return bf16_bits_to_f32(bits).astype(np.float64)


def zipf_probabilities(C: int, s: float) -> np.ndarray:
    w = np.arange(1, C + 1, dtype=np.float64) ** (-float(s))
    return w / w.sum()


def draw_labels(rng: np.random.Generator, B: int, C: int, dist) -> np.ndarray:
    if dist == "uniform":
        return rng.integers(0, C, size=B, dtype=np.int64).astype(np.int32)
    kind, s = dist
    if kind != "zipf":
        raise ValueError(f"unknown label distribution {dist!r}")
    return rng.choice(C, size=B, p=zipf_probabilities(C, s)).astype(np.int32)


def _draw_normal_bf16(rng, rows, cols, sigma, relu, chunk_rows=8192):
    out = np.empty((rows, cols), dtype=np.uint16)
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        v = rng.standard_normal((r1 - r0, cols), dtype=np.float32)
        if sigma != 1.0:
            v *= np.float32(sigma)
        if relu:
            np.maximum(v, np.float32(0.0), out=v)
        out[r0:r1] = f32_to_bf16_bits(v)
    return out


@dataclass
class SplitFcInputs:
    """One seeded problem instance. W_bits holds classes [w_lo, w_lo + W_bits.shape[0])."""
    name: str
    B: int
    D: int
    C: int                       # total classes the labels range over
    X_bits: np.ndarray           # [B, D] uint16 (bf16)
    W_bits: np.ndarray           # [C_w, D] uint16 (bf16), class-major
    bias: Optional[np.ndarray]   # [C_w] float32 or None (= zero)
    labels: np.ndarray           # [B] int32, global class ids
    shards: List[Tuple[int, int]] = field(default_factory=list)   # (class_offset, C_shard)
    w_lo: int = 0


def make_inputs(name, B, D, C, *, x_sigma=1.0, x_relu=False, w_sigma=0.02, labels="uniform",
                shards=None, seed=0, bias_sigma=None, w_rows=None, draw_discarded=True) -> SplitFcInputs:
    """Draw X [B, D], W [C, D] (or only its first `w_rows` classes), labels [B].

    `w_rows` lets a test keep only the leading classes of a very wide layer (the
    remaining rows are still drawn and discarded so the stream position of the
    labels does not depend on it; with `draw_discarded=False` they are skipped,
    which saves a minute for a 1M-class layer and makes the labels depend on `w_rows`).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    X_bits = _draw_normal_bf16(rng, B, D, x_sigma, x_relu)
    keep = C if w_rows is None else int(w_rows)
    W_bits = np.empty((keep, D), dtype=np.uint16)
    chunk = 8192
    for r0 in range(0, C if draw_discarded else keep, chunk):
        r1 = min(C, r0 + chunk)
        blk = _draw_normal_bf16(rng, r1 - r0, D, w_sigma, False)
        if r0 < keep:
            k1 = min(keep, r1)
            W_bits[r0:k1] = blk[: k1 - r0]
    y = draw_labels(rng, B, C, labels)
    bias = None
    if bias_sigma is not None:
        bias = (rng.standard_normal(keep, dtype=np.float32) * np.float32(bias_sigma)).astype(np.float32)
    if shards is None:
        shards = [(0, C)]
    return SplitFcInputs(name, B, D, C, X_bits, W_bits, bias, y, list(shards), 0)


def equal_shards(C: int, n: int) -> List[Tuple[int, int]]:
    assert C % n == 0
    w = C // n
    return [(i * w, w) for i in range(n)]


# The five workload configurations plus the headline shape.  `timed_shards` are the
# shards one bench step runs; `shards` are the ones parity runs and combines.
CONFIGS = {
    # tiny CPU-checkable case
    "cfg1": dict(B=32, D=256, C=1000, x_sigma=0.02, w_sigma=0.02, labels="uniform",
                 shards=equal_shards(1000, 2)),
    # the paper's classifier, unsharded
    "cfg2": dict(B=256, D=2048, C=100_000, x_relu=True, w_sigma=0.01, labels="uniform",
                 shards=[(0, 100_000)]),
    # one GPU's equal share (8-way), all shards run one after another and combined
    "cfg3": dict(B=1024, D=2048, C=100_000, x_relu=True, w_sigma=0.01, labels="uniform",
                 shards=equal_shards(100_000, 8)),
    # hardware-aware uneven partition: two fast and two slow devices at 3:1
    "cfg4": dict(B=1024, D=2048, C=100_000, x_relu=True, w_sigma=0.01, labels=("zipf", 1.1),
                 shards=[(0, 37_500), (37_500, 12_500), (50_000, 37_500), (87_500, 12_500)]),
    # large-vocabulary head: first 50 000 of 400 000 classes
    "cfg5": dict(B=8192, D=1024, C=400_000, x_sigma=1.0, w_sigma=0.02, labels=("zipf", 1.0),
                 shards=equal_shards(400_000, 8)),
    # the paper's second workload: a 1M-class layer cut 8 ways (Section 5.1.2, the 1M-class hybrid run)
    "million": dict(B=1024, D=2048, C=1_000_000, x_relu=True, w_sigma=0.01, labels="uniform",
                    shards=equal_shards(1_000_000, 8), draw_discarded=False),
    # headline shape: the whole 100K-class layer as one shard at B = 1024
    "headline": dict(B=1024, D=2048, C=100_000, x_relu=True, w_sigma=0.01, labels="uniform",
                     shards=[(0, 100_000)]),
}


def make_config(name: str, seed: int = 0, w_rows=None) -> SplitFcInputs:
    kw = dict(CONFIGS[name])
    return make_inputs(name, kw.pop("B"), kw.pop("D"), kw.pop("C"), seed=seed, w_rows=w_rows, **kw)
