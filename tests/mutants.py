"""Planted mistakes for the study of the probabilistic test (Sec. 4.2, Sec. 5.2, Fig. 2): how many
random samples does it take until a wrong kernel is caught?

TEST INFRASTRUCTURE, CPU only.  Nothing wrong is ever run on the GPU: the mistakes are planted
in a plain numpy float64 model of the method under test (tiled attention with online softmax,
the steps of the hot path in their order), and each mutant is compared with the fp64 oracle
on random inputs exactly as a kernel would be.  `tiled_attention(..., bug=None)` is the
correct method and agrees with the oracle to rounding.
"""
from __future__ import annotations

import numpy as np

BN = 64  # keys per tile of the model (the shipped default)

# name -> (what is wrong, when it can show)
BUGS = {
    "tail_key_dropped": ("the last key of a ragged last tile is masked out", "N not a multiple of the tile"),
    "no_rescale_of_O": ("when the running maximum rises, l is rescaled but O is not", "a later tile holds a larger score"),
    "diag_first_key": ("causal mask hides key == query when the key is the first of its tile", "causal, N > tile"),
    "stale_v_tile": ("odd tiles multiply P with the V tile before them (a buffer that was not refilled)", "N > tile"),
    "lse_in_base_2": ("lse is returned as log2 of the sum instead of ln", "always, unless lse is ~0"),
    "mask_after_max": ("the running maximum is taken before the causal mask is applied", "causal; benign for O, lse unaffected"),
    "first_tile_only_max": ("the reference maximum is never raised after the first tile",
                            "scores so far above the first tile's that exp overflows (hundreds, in this float64 model)"),
    "p_sum_after_rounding": ("the row sum is taken over P rounded to bf16", "short rows; about 1e-3 in lse"),
    "scale_rounded_to_half": ("the scale is rounded to binary16", "d = 128 only (1/sqrt(64) is exact)"),
}


def _round_bf16(x: np.ndarray) -> np.ndarray:
    u = x.astype(np.float32).view(np.uint32)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.view(np.float32).astype(np.float64)


def tiled_attention(q, k, v, causal: bool, scale: float, bug: str | None = None):
    """q, k, v: float64 [N, d] of ONE head.  Returns (O [N, d], lse [N]).  One query row at a time,
    keys in tiles of BN: S = q.K^T * scale, mask, m' = max(m, rowmax), P = exp(S - m'),
    l = l * exp(m - m') + sum(P), O = O * exp(m - m') + P.V; at the end O / l and m + ln l."""
    N, d = q.shape
    O = np.zeros((N, d))
    lse = np.zeros(N)
    if bug == "scale_rounded_to_half":
        scale = float(np.float16(scale))
    ntiles = (N + BN - 1) // BN
    for i in range(N):
        m, l, acc = -np.inf, 0.0, np.zeros(d)
        last = i if causal else N - 1
        for t in range(ntiles):
            k0 = t * BN
            if k0 > last:
                break
            k1 = min(N, k0 + BN)
            s = (k[k0:k1] @ q[i]) * scale
            idx = np.arange(k0, k1)
            visible = idx <= last
            if bug == "tail_key_dropped" and k1 == N and N % BN != 0:
                visible = visible & (idx != N - 1)
            if bug == "diag_first_key" and causal and i == k0 and k0 > 0:
                visible = visible & (idx != i)
            raw_max = s.max()
            s = np.where(visible, s, -np.inf)
            tile_max = raw_max if bug == "mask_after_max" else s.max()
            m_new = max(m, tile_max) if not (bug == "first_tile_only_max" and t > 0) else m
            if not np.isfinite(m_new):
                continue
            with np.errstate(over="ignore", invalid="ignore"):
                p = np.exp(s - m_new)
                alpha = np.exp(m - m_new) if np.isfinite(m) else 0.0
            vt = v[k0:k1]
            if bug == "stale_v_tile" and t % 2 == 1 and k1 - k0 == BN:
                vt = v[k0 - BN:k0]
            psum = _round_bf16(p).sum() if bug == "p_sum_after_rounding" else p.sum()
            l = l * alpha + psum
            acc = (acc if bug == "no_rescale_of_O" else acc * alpha) + p @ vt
            m = m_new
        with np.errstate(divide="ignore", invalid="ignore"):
            O[i] = acc / l
            lse[i] = m + (np.log2(l) if bug == "lse_in_base_2" else np.log(l))
    return O, lse
