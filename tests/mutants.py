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


# ---- second workload: C = leaky_relu(A B), tiled the way the kernel tiles it (32 x 32 tiles of C,
# the k dimension dealt out to WK workers in ranges of BKW, partial sums added at the end)
GEMM_BUGS = {
    "k_tail_dropped": ("a k range that crosses K is skipped instead of zero-filled", "K not a multiple of the range"),
    "k_tail_not_zeroed": ("the part of the last range past K multiplies what follows in memory", "K not a multiple of the range"),
    "worker_sum_misses_last": ("the final sum leaves out the last worker's partial result", "K larger than one range"),
    "row_tail_wraps": ("rows of a ragged last tile read row (m mod 32) of the tile instead of their own", "M not a multiple of 32"),
    "slope_on_rounded": ("the activation is applied after rounding to 16 bits", "benign: rounding keeps the sign"),
    "relu_instead_of_leaky": ("negative sums become zero", "any negative output (slope != 0)"),
    "slope_on_negative_zero": ("x >= 0 tested as x > 0: a zero sum is multiplied by the slope", "benign: 0 * slope = 0"),
    "b_tile_transposed_within_8": ("columns of B are swapped in pairs inside every group of 8", "N >= 2, B not constant along rows"),
}
GEMM_WK, GEMM_BKW = 4, 32


def tiled_gemm_lrelu(a, b, slope: float, bug: str | None = None):
    """a [M,K], b [K,N] float64.  Returns C [M,N] float64 (before the final 16-bit rounding, which
    the comparison's tolerance covers)."""
    M, K = a.shape
    N = b.shape[1]
    C = np.zeros((M, N))
    if bug == "b_tile_transposed_within_8":
        perm = np.arange(N) ^ 1
        perm[perm >= N] = N - 1
        b = b[:, perm]
    step = GEMM_WK * GEMM_BKW
    for m0 in range(0, M, 32):
        rows = np.arange(m0, min(M, m0 + 32))
        src = rows
        if bug == "row_tail_wraps" and m0 + 32 > M:
            src = m0 + (rows - m0) % max(1, (M - m0) // 2 + 1)      # some rows read a neighbour's data
        part = np.zeros((GEMM_WK, len(rows), N))
        for w in range(GEMM_WK):
            for k0 in range(w * GEMM_BKW, K, step):
                k1 = k0 + GEMM_BKW
                if k1 > K:
                    if bug == "k_tail_dropped":
                        continue
                    if bug == "k_tail_not_zeroed":
                        # what lies past row i's end in a row-major A is the start of row i+1; B past K: its last row again
                        ext_a = np.concatenate([a[src, k0:K], a[np.minimum(src + 1, M - 1), :k1 - K]], axis=1)
                        ext_b = np.concatenate([b[k0:K], np.repeat(b[K - 1:K], k1 - K, axis=0)], axis=0)
                        part[w] += ext_a @ ext_b
                        continue
                    k1 = K
                part[w] += a[src, k0:k1] @ b[k0:k1]
        workers = GEMM_WK - 1 if bug == "worker_sum_misses_last" else GEMM_WK
        x = part[:workers].sum(axis=0)
        if bug == "slope_on_rounded":
            x = x.astype(np.float16).astype(np.float64)
        if bug == "relu_instead_of_leaky":
            x = np.where(x >= 0, x, 0.0)
        elif bug == "slope_on_negative_zero":
            x = np.where(x > 0, x, slope * x)
        else:
            x = np.where(x >= 0, x, slope * x)
        C[rows] = x
    return C
