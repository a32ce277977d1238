"""GPU parity: the HIP path (through the C-ABI binding) against the CPU oracle,
element by element on the same seeded inputs."""
import numpy as np
import pytest

from oracle import ref
from paper_2403_16863_amd import inputs as I

from gpu_util import check, run_gpu

pytestmark = pytest.mark.gpu


def variants_for(d, dtype, causal):
    import paper_2403_16863_amd as A
    return [v for v in range(A.attn_num_variants()) if A.attn_variant_supported(v, d, dtype, causal)]


SMALL_N = (1, 2, 17, 31, 32, 33, 64, 65, 127, 128, 129, 200, 257, 383, 1000)


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
def test_small_shapes_all_variants(d, causal, dtype):
    """Sizes the oracle finishes in seconds, spanning several tiles and ragged tails."""
    for N in SMALL_N:
        w = I.Workload("t", 2, 3, N, d, causal, dtype)
        qb, kb, vb = I.make_qkv(w, seed=1000 + N)
        O_ref, l_ref, _ = ref.attn_ref(qb, kb, vb, causal, w.scale, dtype)
        for var in [None] + variants_for(d, dtype, causal):
            print(f"case N={N} d={d} causal={causal} dtype={dtype} variant={var}", flush=True)
            O, l = run_gpu(qb, kb, vb, causal, w.scale, dtype, variant=var)
            check(O, l, O_ref, l_ref, dtype, what=f"N={N} d={d} causal={causal} dt={dtype} var={var}")


@pytest.mark.parametrize("idx", [0, 1])
def test_benchmark_configs_full(idx):
    """cfg0 and cfg1 are small enough for the full oracle."""
    w = I.WORKLOADS[idx]
    qb, kb, vb = I.make_qkv(w, seed=idx)
    O_ref, l_ref, _ = ref.attn_ref(qb, kb, vb, w.causal, w.scale, w.dtype)
    for var in [None] + variants_for(w.d, w.dtype, w.causal):
        print(f"case {w.label} variant={var}", flush=True)
        O, l = run_gpu(qb, kb, vb, w.causal, w.scale, w.dtype, variant=var)
        check(O, l, O_ref, l_ref, w.dtype, what=f"{w.label} var={var}")


def boundary_and_round_rows(w, bm=256):
    """Rows the launch configuration makes special: both sides of every query-tile boundary of
    one head (first, last and the rows next to them of every tile), and rows of the work items
    that the first and the last workgroup take in every round of the persistent schedule."""
    import paper_2403_16863_amd as A
    rows = set()
    nqt = (w.N + bm - 1) // bm
    head = (w.B * w.H) // 2
    for t in range(nqt):
        for i in (t * bm, t * bm + 1, t * bm + bm // 2, min(w.N, (t + 1) * bm) - 2, min(w.N, (t + 1) * bm) - 1):
            if 0 <= i < w.N:
                rows.add(head * w.N + i)
    var = A.attn_default_variant(w.N, w.d, w.dtype, w.causal)
    grid = A.attn_schedule_grid(var, 256, w.B, w.H, w.N)
    for wg in (0, grid // 2, grid - 1):
        rnd = 0
        while True:
            item = A.attn_schedule_item(grid, wg, w.B * w.H, nqt, rnd)
            if item is None:
                break
            bh, qt = item
            for i in (qt * bm, qt * bm + 33, min(w.N, (qt + 1) * bm) - 1):
                if i < w.N:
                    rows.add(bh * w.N + i)
            rnd += 1
    return rows


@pytest.mark.parametrize("idx,nrows", [(2, 8192), (3, 16384), (4, 4096)])
def test_benchmark_configs_sampled(idx, nrows):
    """Full-size workloads in the launch configuration bench.py times, compared on
    sampled rows the oracle computes one by one (random rows of every head, both sides of every
    query-tile boundary of one head, rows of every round of the schedule); every output must
    be finite."""
    w = I.WORKLOADS[idx]
    qb, kb, vb = I.make_qkv(w, seed=idx)
    rows = set(int(r) for r in I.sample_rows(w, nrows, seed=idx))
    rows |= boundary_and_round_rows(w, 256 if w.d == 128 else 128)
    rows = np.array(sorted(rows), dtype=np.int64)
    O_ref, l_ref, _ = ref.attn_ref(qb, kb, vb, w.causal, w.scale, w.dtype, rows=rows)
    print(f"case {w.label} default variant", flush=True)
    O, l = run_gpu(qb, kb, vb, w.causal, w.scale, w.dtype)
    check(O.reshape(-1, w.d)[rows], l.reshape(-1)[rows], O_ref, l_ref, w.dtype, what=w.label)
    assert np.isfinite(O).all() and np.isfinite(l).all()
    # property that holds at any size: outputs are convex combinations of V rows
    v = I.bits_to_f64(vb, w.dtype)
    vmax = np.abs(v).max(axis=2, keepdims=True)
    assert (np.abs(O) <= vmax * (1 + 1e-2) + 1e-3).all()


@pytest.mark.parametrize("B,H,N,d,causal,dtype,nrows", [
    (1, 1, 65536, 128, True, I.BF16, 3072),     # one very long sequence: 256 query tiles of one head
    (1, 2, 40000, 64, False, I.F16, 192),       # long, ragged (40000 = 625 * 64), no mask
    (64, 64, 64, 64, True, I.F16, 1024),        # 4096 heads of one tile each: more work items than workgroups
    (3, 37, 257, 128, True, I.BF16, 1024),      # head count without a factor of 8, one row past a tile
    (1, 1000, 1, 64, False, I.BF16, 1000),      # a thousand single-key heads
    (2, 3, 4100, 64, True, I.BF16, 512),        # long causal d = 64 (three workgroups per CU), ragged tail
])
def test_extreme_shapes_sampled(B, H, N, d, causal, dtype, nrows):
    """Shapes at the ends of what the schedule has to deal out (very long heads, very many heads,
    head counts that do not divide over the XCDs), compared on sampled rows; every output finite."""
    w = I.Workload("extreme", B, H, N, d, causal, dtype)
    qb, kb, vb = I.make_qkv(w, seed=N)
    rows = set(int(r) for r in I.sample_rows(w, nrows, seed=N))
    if N >= 4096:
        rows |= boundary_and_round_rows(w, 256 if d == 128 else 128)
    rows = np.array(sorted(rows), dtype=np.int64)
    O_ref, l_ref, _ = ref.attn_ref(qb, kb, vb, w.causal, w.scale, w.dtype, rows=rows)
    print(f"case {w.label} default variant", flush=True)
    O, l = run_gpu(qb, kb, vb, w.causal, w.scale, w.dtype)
    check(O.reshape(-1, w.d)[rows], l.reshape(-1)[rows], O_ref, l_ref, w.dtype, what=w.label)
    assert np.isfinite(O).all() and np.isfinite(l).all()


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("kind", I.ADVERSARIAL)
def test_adversarial_inputs(kind, dtype):
    for (N, d, causal) in ((129, 64, False), (200, 128, True), (64, 128, False)):
        qb, kb, vb = I.make_adversarial(kind, 1, 2, N, d, dtype, seed=7)
        scale = float(np.float32(1.0 / np.sqrt(d)))
        O_ref, l_ref, _ = ref.attn_ref(qb, kb, vb, causal, scale, dtype)
        out_scale = max(1.0, float(np.abs(I.bits_to_f64(vb, dtype)).max()))
        for var in [None] + variants_for(d, dtype, causal):
            print(f"case {kind} N={N} d={d} causal={causal} dtype={dtype} variant={var}", flush=True)
            O, l = run_gpu(qb, kb, vb, causal, scale, dtype, variant=var)
            check(O, l, O_ref, l_ref, dtype, out_scale=out_scale, what=f"{kind} var={var}")


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("d", [64, 128])
def test_reference_maximum_raised_in_mid_stream_all_variants(d, dtype):
    """Scores that climb by dozens from the first key to the last, tile after tile, with a peak on
    the last key: every variant has to raise its reference maximum in the middle of the key
    stream and at its end (for the interleaved and the two-cluster orders that path sits inside
    the pipelined MFMA streams), with and without the causal mask, past several tiles."""
    for N, causal in ((512, False), (640, True), (1100, False), (1100, True)):
        qb, kb, vb = I.make_adversarial("rising_scores", 1, 2, N, d, dtype, seed=N + d)
        scale = float(np.float32(1.0 / np.sqrt(d)))
        O_ref, l_ref, _ = ref.attn_ref(qb, kb, vb, causal, scale, dtype)
        out_scale = max(1.0, float(np.abs(I.bits_to_f64(vb, dtype)).max()))
        for var in [None] + variants_for(d, dtype, causal):
            print(f"case rising N={N} d={d} causal={causal} dtype={dtype} variant={var}", flush=True)
            O, l = run_gpu(qb, kb, vb, causal, scale, dtype, variant=var)
            check(O, l, O_ref, l_ref, dtype, out_scale=out_scale, what=f"rising N={N} causal={causal} var={var}")


@pytest.mark.parametrize("dtype,vlim", [(I.F16, 10.0), (I.BF16, 3.75)])
def test_accuracy_bound_at_the_stated_limit(dtype, vlim):
    """The header's accuracy bound: the error is at most about 2 u Vmax (u = 2^-11 binary16, 2^-8
    bfloat16), so the absolute tolerances hold for |V| up to 10 / 3.8 even when a row puts all its
    weight on values of that size and one sign (rounding of P and the final rounding then add up).
    Also the V magnitude limit: bfloat16 values of 2^110 with N = 129 keys stay finite and accurate
    relative to their size."""
    g = np.random.Generator(np.random.Philox(key=np.array([77, 5], dtype=np.uint64)))
    for d, N, causal in ((128, 300, True), (64, 257, False), (128, 1000, False)):
        shape = (1, 2, N, d)
        q = g.standard_normal(shape, dtype=np.float32)
        k = g.standard_normal(shape, dtype=np.float32)
        v = (np.float32(vlim) * (np.float32(0.93) + np.float32(0.07) * g.random(shape, dtype=np.float32))).astype(np.float32)
        qb, kb, vb = (I.f32_to_bits(x, dtype) for x in (q, k, v))
        scale = float(np.float32(1.0 / np.sqrt(d)))
        O_ref, l_ref, _ = ref.attn_ref(qb, kb, vb, causal, scale, dtype)
        for var in [None] + variants_for(d, dtype, causal):
            print(f"case bound |v|<={vlim} N={N} d={d} causal={causal} dtype={dtype} variant={var}", flush=True)
            O, l = run_gpu(qb, kb, vb, causal, scale, dtype, variant=var)
            check(O, l, O_ref, l_ref, dtype, what=f"|v|<={vlim} N={N} var={var}")
            u = 2.0 ** -11 if dtype == I.F16 else 2.0 ** -8
            assert np.max(np.abs(O - O_ref)) <= 2.05 * u * vlim, "outside the derived bound 2 u Vmax"
    big = np.float32(2.0 ** 110)
    shape = (1, 2, 129, 128)
    q = g.standard_normal(shape, dtype=np.float32)
    k = g.standard_normal(shape, dtype=np.float32)
    v = np.where(g.random(shape, dtype=np.float32) < 0.5, big, -big).astype(np.float32)
    qb, kb, vb = (I.f32_to_bits(x, I.BF16) for x in (q, k, v))
    scale = float(np.float32(1.0 / np.sqrt(128)))
    O_ref, l_ref, _ = ref.attn_ref(qb, kb, vb, False, scale, I.BF16)
    O, l = run_gpu(qb, kb, vb, False, scale, I.BF16)
    check(O, l, O_ref, l_ref, I.BF16, out_scale=float(big), what="V = +-2^110")


def test_scale_argument_and_stream():
    """Non-default scale, and a launch on a side stream."""
    import torch
    import paper_2403_16863_amd as A
    from gpu_util import to_device
    # (a zero and a negative scale take their own paths where Q enters the registers: q' = 0, q' = -q;
    # both the staged and the direct form of that are covered: d = 128 ping-pong, d = 64, and variant 0)
    for w2, variant in ((I.Workload("t", 1, 2, 300, 64, True, I.F16), None), (I.Workload("t", 1, 2, 300, 128, True, I.BF16), None),
                        (I.Workload("t", 2, 1, 200, 128, False, I.BF16), 0)):
        qb, kb, vb = I.make_qkv(w2, seed=5)
        for scale in (0.0, 0.03, 0.5, -0.2):
            O_ref, l_ref, _ = ref.attn_ref(qb, kb, vb, w2.causal, float(np.float32(scale)), w2.dtype)
            O, l = run_gpu(qb, kb, vb, w2.causal, scale, w2.dtype, variant=variant)
            check(O, l, O_ref, l_ref, w2.dtype, what=f"scale={scale} d={w2.d} variant={variant}")
    w = I.Workload("t", 1, 2, 300, 64, True, I.F16)
    qb, kb, vb = I.make_qkv(w, seed=5)
    s = torch.cuda.Stream()
    q, k, v = (to_device(a, I.F16) for a in (qb, kb, vb))
    out = torch.empty_like(q)
    lse = torch.empty(q.shape[:3], dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    A.attn_fwd(q, k, v, out, lse, True, w.scale, stream=s.cuda_stream)
    s.synchronize()
    O_ref, l_ref, _ = ref.attn_ref(qb, kb, vb, True, w.scale, I.F16)
    check(out.double().cpu().numpy(), lse.double().cpu().numpy(), O_ref, l_ref, I.F16, what="side stream")


def test_errors_leave_outputs_untouched():
    import torch
    import paper_2403_16863_amd as A
    q = torch.zeros(1, 1, 8, 64, dtype=torch.float16, device="cuda")
    out = torch.full_like(q, 3.0)
    lse = torch.full((1, 1, 8), 5.0, dtype=torch.float32, device="cuda")
    with pytest.raises(A.AttnError) as e:
        A.attn_fwd(q, q, q, q, lse, False, 1.0)            # out aliases q
    assert e.value.code == -1
    with pytest.raises(A.AttnError):
        A.attn_fwd(q, q, q, out, lse, False, float("nan"))
    with pytest.raises(A.AttnError):
        A.attn_fwd_variant(q, q, q, out, lse, False, 1.0, A.attn_num_variants())
    torch.cuda.synchronize()
    assert (out == 3.0).all() and (lse == 5.0).all()
