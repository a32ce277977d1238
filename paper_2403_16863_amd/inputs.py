"""Seeded synthetic Q/K/V for the attention-forward workloads.

This module only *makes inputs*: it draws numbers from a counter-based generator
(numpy's Philox), rounds them to 16-bit floating point on the host and hands out
the raw bit patterns.  It holds none of the attention arithmetic and imports
neither the GPU binding nor the CPU oracle; both are fed the same bit patterns.

The paper's own workload is a shape filled with random tensors
([batch, heads, seq, head_dim], half precision; Table 2 caption and Sec. 4.2), so
random tensors of LLM-attention shapes stand in for it here.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

F16 = 0
BF16 = 1
DTYPE_NAMES = {F16: "f16", BF16: "bf16"}


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int
    d: int
    causal: bool
    dtype: int
    qk_sigma: float = 1.0      # Q and K are iid N(0, qk_sigma^2)
    v_dist: str = "normal"     # "normal": N(0,1); "uniform": U(-1,1)

    @property
    def scale(self) -> float:
        """1/sqrt(d) rounded to fp32: the value handed to the GPU and, widened
        exactly to fp64, to the oracle."""
        return float(np.float32(1.0) / np.sqrt(np.float32(self.d)))

    @property
    def flops(self) -> float:
        """Customary count: 4*B*H*N^2*d, halved when causal."""
        f = 4.0 * self.B * self.H * self.N * self.N * self.d
        return f / 2 if self.causal else f

    @property
    def label(self) -> str:
        return (f"{self.name}: B{self.B} H{self.H} N{self.N} d{self.d} "
                f"{'causal' if self.causal else 'full'} {DTYPE_NAMES[self.dtype]}")


# The five benchmark configurations (index = position in the configs list).
WORKLOADS = (
    Workload("cfg0", 1, 2, 128, 64, False, F16),
    Workload("cfg1", 4, 16, 1024, 64, True, F16),
    Workload("cfg2", 2, 32, 4096, 128, True, BF16),
    Workload("cfg3", 1, 32, 16384, 128, True, BF16),
    Workload("cfg4", 8, 16, 2048, 64, False, F16, qk_sigma=2.0, v_dist="uniform"),
)


def f32_to_bits(x: np.ndarray, dtype: int) -> np.ndarray:
    """Round float32 values to nearest-even 16-bit patterns (uint16)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == F16:
        return x.astype(np.float16).view(np.uint16)
    if dtype == BF16:
        u = x.view(np.uint32)
        # nearest-even: add 0x7fff plus the lowest kept bit, then truncate
        rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
        out = rounded.astype(np.uint16)
        nan = np.isnan(x)
        if nan.any():
            out[nan] = 0x7FC0
        return out
    raise ValueError(f"unknown dtype {dtype}")


def bits_to_f64(bits: np.ndarray, dtype: int) -> np.ndarray:
    """Exact widening of 16-bit patterns to float64 using numpy's own types."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == F16:
        return bits.view(np.float16).astype(np.float64)
    if dtype == BF16:
        with np.errstate(invalid="ignore"):   # signalling-NaN patterns widen quietly
            return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype}")


def _rng(seed: int, stream: int) -> np.random.Generator:
    key = np.array([seed & 0xFFFFFFFFFFFFFFFF, stream], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def make_qkv(w: Workload, seed: int):
    """Return (q, k, v) as uint16 arrays of shape [B,H,N,d] holding 16-bit patterns."""
    shape = (w.B, w.H, w.N, w.d)
    q = _rng(seed, 0).standard_normal(shape, dtype=np.float32)
    k = _rng(seed, 1).standard_normal(shape, dtype=np.float32)
    if w.qk_sigma != 1.0:
        q *= np.float32(w.qk_sigma)
        k *= np.float32(w.qk_sigma)
    if w.v_dist == "normal":
        v = _rng(seed, 2).standard_normal(shape, dtype=np.float32)
    elif w.v_dist == "uniform":
        v = _rng(seed, 2).random(shape, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)
    else:
        raise ValueError(w.v_dist)
    return f32_to_bits(q, w.dtype), f32_to_bits(k, w.dtype), f32_to_bits(v, w.dtype)


# Adversarial families used by the randomized admission tests.  Each returns
# float32 arrays that are then rounded like the ordinary inputs.
ADVERSARIAL = ("peaked", "equal_scores", "large_negative", "single_v_row", "signed_zero",
               "max_finite_v", "rising_scores")


def make_adversarial(kind: str, B: int, H: int, N: int, d: int, dtype: int, seed: int):
    shape = (B, H, N, d)
    g = _rng(seed, 7)
    q = g.standard_normal(shape, dtype=np.float32)
    k = g.standard_normal(shape, dtype=np.float32)
    v = g.standard_normal(shape, dtype=np.float32)
    if kind == "peaked":
        # one key per head points 8x along a query direction: a near one-hot row
        j = int(g.integers(0, N))
        i = int(g.integers(0, N))
        k[:, :, j, :] = 8.0 * q[:, :, i, :]
    elif kind == "equal_scores":
        k[:] = k[:, :, :1, :]            # all keys identical: uniform softmax
    elif kind == "large_negative":
        k[:] = -np.abs(k) * 6.0
        q[:] = np.abs(q) * 6.0           # every score strongly negative
    elif kind == "single_v_row":
        j = int(g.integers(0, N))
        keep = v[:, :, j, :].copy()
        v[:] = 0.0
        v[:, :, j, :] = keep
    elif kind == "signed_zero":
        mask = g.random(shape, dtype=np.float32) < 0.5
        q[mask] = -0.0
        k[~mask] = 0.0
    elif kind == "max_finite_v":
        # binary16: the largest finite value.  bfloat16: 2^100 -- the one-pass method
        # keeps the un-normalised sum of p*v in fp32, so |v| * N has to stay below the
        # fp32 range; the largest finite bfloat16 (3.4e38) cannot be averaged that way.
        big = 65504.0 if dtype == F16 else 2.0 ** 100
        v[:] = np.where(g.random(shape, dtype=np.float32) < 0.5, big, -big).astype(np.float32)
    elif kind == "rising_scores":
        # every query scores key j at about 3 * sqrt(d) * j / N (scaled by 1/sqrt(d)) plus noise: the
        # scores climb by dozens over the sequence, tile after tile, and the last key is a peak on
        # top.  A one-pass softmax has to move its reference maximum again and again, in the
        # middle of the key stream and at its end.
        u = g.standard_normal(d, dtype=np.float32)
        u /= np.float32(np.linalg.norm(u))
        root = np.float32(np.sqrt(d))
        q[:] = q * np.float32(0.25) + u * root
        ramp = (np.arange(N, dtype=np.float32) / np.float32(max(N, 1)))[None, None, :, None]
        k[:] = k * np.float32(0.25) + np.float32(3.0) * ramp * u * root
        k[:, :, N - 1, :] += np.float32(1.5) * u * root
    else:
        raise ValueError(kind)
    return f32_to_bits(q, dtype), f32_to_bits(k, dtype), f32_to_bits(v, dtype)


def sample_rows(w: Workload, count: int, seed: int, edges=(31, 32, 63, 64, 127, 128, 255, 256)):
    """Flattened (b*H+h)*N+i row indices: first and last row, rows around tile
    edges, and uniformly drawn rows, spread over all heads.  Sorted by head."""
    g = _rng(seed, 11)
    bh_n = w.B * w.H
    rows = set()
    for bh in {0, bh_n - 1, int(g.integers(0, bh_n))}:
        for i in (0, 1, w.N - 1, w.N - 2, w.N // 2, *edges):
            if 0 <= i < w.N:
                rows.add(bh * w.N + i)
    total = bh_n * w.N
    count = min(count, total)
    while len(rows) < count:
        need = count - len(rows)
        rows.update(int(r) for r in g.integers(0, total, size=need))
    return np.array(sorted(rows), dtype=np.int64)


# ---- second workload: fused GEMM + LeakyReLU (Sec. 5, Table 3).  The paper's input is a shape
# (M, N, K = 512, 512, 2048, binary16) filled with random tensors; the slope is not stated.
GEMM_M, GEMM_N, GEMM_K = 512, 512, 2048
GEMM_SLOPE = 0.01
GEMM_FAMILIES = ("normal", "positive", "cancelling", "signed_zero", "large", "one_hot")


def make_gemm(M: int, N: int, K: int, dtype: int, seed: int, family: str = "normal"):
    """Return (a [M,K], b [K,N]) as uint16 bit patterns.  "normal": iid N(0,1), the sum over K then
    has both signs, so both branches of the activation are taken.  The other families stress
    one thing each: "positive" (no negative output), "cancelling" (pairs of equal and opposite
    products: outputs near zero from large terms), "signed_zero" (half of the entries +-0),
    "large" (entries scaled by 8: sums near the top of binary16's range), "one_hot" (each row of A has
    a single 1: C is a row gather of B, exact)."""
    g = _rng(seed, 21)
    a = g.standard_normal((M, K), dtype=np.float32)
    b = g.standard_normal((K, N), dtype=np.float32)
    if family == "normal":
        pass
    elif family == "positive":
        a, b = np.abs(a), np.abs(b)
    elif family == "cancelling":
        h = K // 2
        if h:
            a[:, h:2 * h] = -a[:, :h] * np.float32(64.0)
            a[:, :h] *= np.float32(64.0)
            b[h:2 * h, :] = b[:h, :]
    elif family == "signed_zero":
        za = g.random((M, K), dtype=np.float32) < 0.5
        zb = g.random((K, N), dtype=np.float32) < 0.5
        a[za] = -0.0
        b[zb] = 0.0
    elif family == "large":
        a *= np.float32(8.0)
        b *= np.float32(8.0)
    elif family == "one_hot":
        a[:] = 0.0
        a[np.arange(M), g.integers(0, K, size=M)] = 1.0
    else:
        raise ValueError(family)
    return f32_to_bits(a, dtype), f32_to_bits(b, dtype)
