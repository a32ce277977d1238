"""The schedule search on the GPU: admission against the oracle for every step's
candidate, and the product's own admission test against the default variant."""
import pytest

from oracle import ref
from paper_2403_16863_amd import inputs as I
from paper_2403_16863_amd import search as S

from gpu_util import check, run_gpu

pytestmark = pytest.mark.gpu


def oracle_admit(variant, d, dtype, causal, seeds=(0, 1, 2)):
    """Sec. 4.2 with the fp64 oracle as the reference output."""
    for seed in seeds:
        for N in (1, 17, 129, 300):
            w = I.Workload("adm", 1, 2, N, d, causal, dtype, qk_sigma=2.0 if seed == 2 else 1.0)
            qb, kb, vb = I.make_qkv(w, seed=5000 + 37 * seed + N)
            O_ref, l_ref, _ = ref.attn_ref(qb, kb, vb, causal, w.scale, dtype)
            O, l = run_gpu(qb, kb, vb, causal, w.scale, dtype, variant=variant)
            try:
                check(O, l, O_ref, l_ref, dtype)
            except AssertionError:
                return False
    return True


def test_anneal_with_oracle_admission_on_small_workload():
    import torch
    import paper_2403_16863_amd as A
    w = I.Workload("s", 2, 8, 1024, 128, True, I.BF16)
    lat = S.Lattice.from_library(w.d, w.dtype, w.causal)
    q, k, v = S._device_inputs(w.B, w.H, w.N, w.d, w.dtype, 99)
    out = torch.empty_like(q)
    lse = torch.empty(q.shape[:3], dtype=torch.float32, device="cuda")
    x0 = tuple(A.attn_variant_coords(A.attn_default_variant(w.N, w.d, w.dtype, w.causal)))
    res = S.anneal(lat, x0,
                   measure=lambda c: S.measure_variant((q, k, v, out, lse), True, w.scale, lat.points[c], 3, 10),
                   admit=lambda c: oracle_admit(lat.points[c], w.d, w.dtype, w.causal),
                   seed=0, t_max=0.05, t_min=0.02, cool=1.05)
    assert len(res.steps) >= 10
    assert not res.rejected, f"variants failed the oracle: {[lat.points[c] for c in res.rejected]}"
    assert res.t_best <= res.t0 and res.best in res.times
    assert res.ranking()[0][1] == min(res.times.values())


def test_product_admission_accepts_every_built_variant():
    import paper_2403_16863_amd as A
    for d, dtype, causal in ((128, I.BF16, True), (64, I.F16, False)):
        for var in range(A.attn_num_variants()):
            if A.attn_variant_supported(var, d, dtype, causal):
                print(f"admit variant {var} d={d} dtype={dtype} causal={causal}", flush=True)
                assert S.admit_against_default(var, d, dtype, causal, samples=48, seed=1)
