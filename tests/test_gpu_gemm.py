"""GPU parity of the fused GEMM + LeakyReLU kernel (Sec. 5, Table 3) with the fp64 oracle, element
by element, through the C ABI.

Tolerance, derived from the arithmetic: the kernel sums the K products in fp32 (any order) and
rounds once to the 16-bit output, so against the exact value x
    |c - x| <= u_out * |x| + 2 K 2^-24 * sum_k |a_k b_k| + (smallest subnormal step),
u_out = 2^-11 (binary16) or 2^-8 (bfloat16), with a 1 % margin on the first term.  The sum of
absolute products comes from the oracle itself, run on |A|, |B| with slope 1.
"""
import numpy as np
import pytest

from oracle import ref
from paper_2403_16863_amd import inputs as I

pytestmark = pytest.mark.gpu

U_OUT = {I.F16: 2.0 ** -11, I.BF16: 2.0 ** -8}
TINY = {I.F16: 2.0 ** -25, I.BF16: 2.0 ** -134}
MAX_FINITE = {I.F16: 65504.0, I.BF16: 3.3e38}


def torch_dtype(dtype):
    import torch
    return torch.float16 if dtype == I.F16 else torch.bfloat16


def to_device(bits, dtype):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to("cuda").view(torch_dtype(dtype))


def run_gpu(ab, bb, slope, dtype, variant=None, pad=64):
    """C as float64 [M,N].  C lives inside a larger buffer filled with NaN patterns: every element of C
    must be overwritten and nothing around it touched."""
    import torch
    from paper_2403_16863_amd import gemm
    M, K = ab.shape
    N = bb.shape[1]
    a, b = to_device(ab, dtype), to_device(bb, dtype)
    buf = torch.full((pad + M * N + pad,), float("nan"), dtype=torch_dtype(dtype), device="cuda")
    c = buf[pad:pad + M * N].view(M, N)
    if variant is None:
        gemm.gemm_lrelu(a, b, c, slope)
    else:
        gemm.gemm_lrelu_variant(a, b, c, slope, variant)
    torch.cuda.synchronize()
    assert bool(torch.isnan(buf[:pad]).all()) and bool(torch.isnan(buf[pad + M * N:]).all()), "wrote outside C"
    return c.to(torch.float64).cpu().numpy()


def check(c, ab, bb, slope, dtype, what):
    slope32 = float(np.float32(slope))
    x, _ = ref.gemm_lrelu_ref(ab, bb, slope32, dtype)
    mask = np.uint16(0x7FFF)
    sabs, _ = ref.gemm_lrelu_ref(ab & mask, bb & mask, 1.0, dtype)
    K = ab.shape[1]
    assert np.abs(x).max() < 0.9 * MAX_FINITE[dtype], f"{what}: test case overflows the output type"
    tol = 1.01 * U_OUT[dtype] * np.abs(x) + 2.0 * K * 2.0 ** -24 * sabs * max(1.0, abs(slope32)) + TINY[dtype]
    assert np.isfinite(c).all(), f"{what}: non-finite output"
    err = np.abs(c - x)
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    assert (err <= tol).all(), f"{what}: |c - x| = {err[worst]:.3e} > {tol[worst]:.3e} at {worst} (x = {x[worst]:.6e})"
    return float((err / tol).max())


def all_variants():
    from paper_2403_16863_amd import gemm
    return range(gemm.gemm_lrelu_num_variants())


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
def test_paper_shape_every_variant(dtype):
    ab, bb = I.make_gemm(I.GEMM_M, I.GEMM_N, I.GEMM_K, dtype, seed=11)
    for v in all_variants():
        c = run_gpu(ab, bb, I.GEMM_SLOPE, dtype, v)
        check(c, ab, bb, I.GEMM_SLOPE, dtype, f"variant {v} dtype {dtype}")
    c = run_gpu(ab, bb, I.GEMM_SLOPE, dtype)
    check(c, ab, bb, I.GEMM_SLOPE, dtype, f"default dtype {dtype}")
    assert (c < 0).any() and (c > 0).any()          # both branches of the activation were taken


RAGGED = [(1, 8, 8), (1, 8, 2048), (31, 24, 40), (33, 40, 72), (32, 32, 32), (64, 64, 64), (100, 72, 136),
          (65, 264, 264), (7, 8, 520), (129, 136, 1000), (96, 520, 24), (257, 96, 776), (40, 1032, 16)]


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
def test_ragged_shapes_every_variant(dtype):
    """Sizes that are not multiples of the 32 x 32 tile, of a wave's k range (32 or 64) or of the
    workgroup's (up to 512), down to a single row and a single 8-wide k step."""
    for n, (M, N, K) in enumerate(RAGGED):
        ab, bb = I.make_gemm(M, N, K, dtype, seed=100 + n)
        for v in all_variants():
            print(f"M{M} N{N} K{K} variant {v} dtype {dtype}", flush=True)
            c = run_gpu(ab, bb, 0.1, dtype, v)
            check(c, ab, bb, 0.1, dtype, f"M{M} N{N} K{K} variant {v} dtype {dtype}")


@pytest.mark.parametrize("family", I.GEMM_FAMILIES)
@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
def test_input_families(family, dtype):
    for (M, N, K) in ((I.GEMM_M, I.GEMM_N, I.GEMM_K), (77, 104, 328)):
        if family == "large" and dtype == I.F16 and K > 1024:
            K = 1024                                  # keeps |sum| inside binary16's range
        ab, bb = I.make_gemm(M, N, K, dtype, seed=5, family=family)
        c = run_gpu(ab, bb, I.GEMM_SLOPE, dtype)
        check(c, ab, bb, I.GEMM_SLOPE, dtype, f"{family} M{M} N{N} K{K} dtype {dtype}")


@pytest.mark.parametrize("slope", [0.0, 1.0, -0.5, 0.01, 2.0, 1e-3])
def test_slopes(slope):
    ab, bb = I.make_gemm(96, 72, 200, I.F16, seed=9)
    c = run_gpu(ab, bb, slope, I.F16)
    check(c, ab, bb, slope, I.F16, f"slope {slope}")
    if slope == 0.0:
        assert (c >= 0).all()


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
def test_one_hot_rows_are_a_bit_exact_gather(dtype):
    """A with a single 1 per row and slope 1/2: every C element is one element of B, or half of it,
    both exactly representable (away from subnormals): the 16-bit patterns must match exactly."""
    M, N, K = 200, 136, 1000
    ab, bb = I.make_gemm(M, N, K, dtype, seed=3, family="one_hot")
    for v in all_variants():
        c = run_gpu(ab, bb, 0.5, dtype, v)
        x, _ = ref.gemm_lrelu_ref(ab, bb, 0.5, dtype)
        big = np.abs(x) > 2.0 ** -10
        assert big.mean() > 0.9
        assert np.array_equal(c[big], x[big]), f"variant {v}"
        assert np.abs(c - x).max() <= 2.0 ** -24


def test_non_finite_inputs_stay_in_their_row_and_column():
    """An infinity in row i of A reaches only row i of C, a NaN in column j of B only column j;
    the zero fill past K never meets them (K = 40 ends inside every variant's k range)."""
    M, N, K = 70, 48, 40
    ab, bb = I.make_gemm(M, N, K, I.F16, seed=4)
    ab, bb = ab.copy(), bb.copy()
    ab[13, 39] = 0x7C00          # +inf
    bb[39, 21] = 0x7E00          # NaN
    x, _ = ref.gemm_lrelu_ref(ab, bb, 0.25, I.F16)
    import torch
    from paper_2403_16863_amd import gemm
    for v in all_variants():
        a, b = to_device(ab, I.F16), to_device(bb, I.F16)
        c = torch.zeros((M, N), dtype=torch.float16, device="cuda")
        gemm.gemm_lrelu_variant(a, b, c, 0.25, v)
        torch.cuda.synchronize()
        c = c.to(torch.float64).cpu().numpy()
        assert np.array_equal(np.isnan(c), np.isnan(x)), f"variant {v}"
        assert np.array_equal(np.isposinf(c), np.isposinf(x)) and np.array_equal(np.isneginf(c), np.isneginf(x))
        fin = np.isfinite(x)
        assert fin.sum() == (M - 1) * (N - 1)
        assert np.abs(c[fin] - x[fin]).max() < 0.05


def test_binding_rejects_what_the_boundary_cannot_take():
    import torch
    from paper_2403_16863_amd import gemm
    a = torch.zeros((32, 64), dtype=torch.float16, device="cuda")
    b = torch.zeros((64, 32), dtype=torch.float16, device="cuda")
    c = torch.zeros((32, 32), dtype=torch.float16, device="cuda")
    with pytest.raises(ValueError):
        gemm.gemm_lrelu(a, b.t(), c, 0.1)                         # not contiguous
    with pytest.raises(ValueError):
        gemm.gemm_lrelu(a, b, c.cpu(), 0.1)
    with pytest.raises(TypeError):
        gemm.gemm_lrelu(a.float(), b.float(), c.float(), 0.1)
    with pytest.raises(gemm.GemmError):
        gemm.gemm_lrelu(a[:, :60].contiguous(), b[:60].contiguous(), c, 0.1)   # K = 60
    with pytest.raises(gemm.GemmError):
        gemm.gemm_lrelu_variant(a, b, c, 0.1, 999)


def test_admission_test_and_a_short_search():
    """Every shipped variant passes the probabilistic test against the default kernel, and a short
    annealing run on the paper's shape ends on an admitted variant that is no slower than the start."""
    from paper_2403_16863_amd import gemm, gemm_search as GS
    for v in all_variants():
        assert GS.admit_against_default(v, I.F16, samples=6, seed=1), f"variant {v}"
    assert GS.admit_against_default(gemm.gemm_lrelu_default_variant(512, 512, 2048), I.BF16, samples=6, seed=2)
    res, table = GS.search(seed=3, cool=1.3)
    assert res.best in table and res.t_best <= res.t0 and len(res.steps) >= 10
    assert not res.rejected


def test_strategy_comparison_runs_on_the_measured_table():
    from paper_2403_16863_amd import search_compare as SC
    label, names, keys, start, measure, admit, unit = SC.gemm_space()
    keys = keys[:6] + [start] if start not in keys[:6] else keys[:6]
    table, rejected = SC.measure_table(keys, measure, admit, reps=3)
    assert not rejected and all(len(v) == 3 and min(v) > 0 for v in table.values())
    res = SC.compare(table, start, budgets=(3, 12), seeds=5)
    assert set(res) == set(SC.STRATEGIES) and all(r["mean_regret"] >= 0 for rows in res.values() for r in rows)
    att = SC.attribution(table, names)
    assert set(att["knobs"]) == set(names)
