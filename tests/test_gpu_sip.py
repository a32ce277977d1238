"""GPU tests of the instruction-level schedule search: the code-object path of the library and
a short annealing run whose winner is checked against the fp64 oracle."""
import math
import shutil
import tempfile

import numpy as np
import pytest

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")]


def _inputs(B, H, N, d, seed):
    import torch
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    mk = lambda: torch.randn(B, H, N, d, device="cuda", generator=g).to(torch.bfloat16)
    return mk(), mk(), mk()


def test_unmodified_code_object_matches_the_library_kernel():
    import torch
    import paper_2403_16863_amd as A
    from paper_2403_16863_amd import sip
    variant = A.attn_default_variant(4096, 128, A.ATTN_BF16, True)
    d = tempfile.mkdtemp(prefix="sip_gpu_")
    try:
        k = sip.Kernel(sip.compile_base(d, 128, A.ATTN_BF16, True, sip.knobs_of_variant(variant)))
        h = A.attn_codeobj_load(sip.assemble(k.render(), d, "same"), k.name, variant, 128, A.ATTN_BF16, True)
        for (B, H, N) in ((1, 2, 100), (2, 8, 1024), (1, 3, 777)):
            q, kk, v = _inputs(B, H, N, 128, N)
            o1, o2 = torch.empty_like(q), torch.full_like(q, float("nan"))
            l1 = torch.empty(B, H, N, dtype=torch.float32, device="cuda")
            l2 = torch.full_like(l1, float("nan"))
            A.attn_fwd_variant(q, kk, v, o1, l1, True, 1 / math.sqrt(128), variant)
            A.attn_fwd_codeobj(h, q, kk, v, o2, l2, True, 1 / math.sqrt(128))
            torch.cuda.synchronize()
            assert torch.equal(o1.view(torch.int16), o2.view(torch.int16)) and torch.equal(l1, l2)
        # a handle refuses shapes it was not loaded for, and bad handles are errors
        q, kk, v = _inputs(1, 1, 64, 64, 1)
        with pytest.raises(A.AttnError):
            A.attn_fwd_codeobj(h, q, kk, v, torch.empty_like(q), torch.empty(1, 1, 64, dtype=torch.float32, device="cuda"),
                               True, 0.125)
        A.attn_codeobj_unload(h)
        with pytest.raises(A.AttnError):
            A.attn_codeobj_unload(h)
        with pytest.raises(A.AttnError):
            A.attn_codeobj_load("/nonexistent.co", k.name, variant, 128, A.ATTN_BF16, True)
    finally:
        shutil.rmtree(d, ignore_errors=True)


def test_short_search_winner_passes_the_oracle():
    import torch
    import paper_2403_16863_amd as A
    from oracle import ref
    from paper_2403_16863_amd import inputs as I
    from paper_2403_16863_amd import sip
    from tests.gpu_util import check
    d = tempfile.mkdtemp(prefix="sip_gpu_")
    try:
        # ~14 annealing steps on the bench workload, then the winner on a ragged causal shape vs the oracle
        out = sip.search_workload(2, seed=3, t_max=0.05, t_min=0.025, cool=1.05, samples=8, keep_best=d + "/best.s",
                                  keep_codeobj=d + "/best.co")
        assert out["steps"] >= 10 and out["admitted"] >= 1
        assert out["best_ms"] <= out["unmodified_codeobj_ms"]
        variant = out["variant"]
        k = sip.Kernel(open(d + "/best.s").read())
        h = A.attn_codeobj_load(sip.assemble(k.render(), d, "best"), k.name, variant, 128, A.ATTN_BF16, True)
        w = I.Workload("sipcheck", 1, 3, 1000, 128, True, I.BF16)
        qb, kb, vb = I.make_qkv(w, 11)
        to = lambda a: torch.from_numpy(a.view(np.int16)).to("cuda").view(torch.bfloat16)
        q, kk, v = to(qb), to(kb), to(vb)
        o = torch.full_like(q, float("nan"))
        l = torch.full((1, 3, 1000), float("nan"), dtype=torch.float32, device="cuda")
        A.attn_fwd_codeobj(h, q, kk, v, o, l, True, w.scale)
        torch.cuda.synchronize()
        O_ref, l_ref, _ = ref.attn_ref(qb, kb, vb, True, w.scale, w.dtype)
        check(o.to(torch.float64).cpu().numpy(), l.to(torch.float64).cpu().numpy(), O_ref, l_ref, w.dtype, what="search winner")
        A.attn_codeobj_unload(h)
        # Sec. 4.1: the kept code object, deployed, is what attn_fwd launches for its shape class,
        # until it is unloaded
        from paper_2403_16863_amd import deploy
        try:
            h2 = deploy.deploy_codeobj_file(d + "/best.co", 1, 100000)
            assert A.attn_deployed(1000, 128, A.ATTN_BF16, True) == (True, variant, h2)
            assert not A.attn_deployed(1000, 128, A.ATTN_BF16, False)[0]
            o2 = torch.full_like(q, float("nan"))
            l2 = torch.full_like(l, float("nan"))
            A.attn_fwd(q, kk, v, o2, l2, True, w.scale)
            torch.cuda.synchronize()
            assert torch.equal(o2.view(torch.int16), o.view(torch.int16)) and torch.equal(l2, l)
            A.attn_codeobj_unload(h2)
            assert not A.attn_deployed(1000, 128, A.ATTN_BF16, True)[0]
            o2.fill_(float("nan"))
            A.attn_fwd(q, kk, v, o2, l2, True, w.scale)       # the library's own kernel again
            torch.cuda.synchronize()
            check(o2.to(torch.float64).cpu().numpy(), l2.to(torch.float64).cpu().numpy(), O_ref, l_ref, w.dtype, what="after unload")
        finally:
            A.attn_deploy_clear()
    finally:
        shutil.rmtree(d, ignore_errors=True)


def test_gemm_code_object_path_and_a_short_search():
    """Second workload: the unmodified kernel loaded from its own assembly reproduces the library
    kernel bit for bit; a short annealing run over instruction positions ends on a kernel that
    passed the test against the unmodified one, and that kernel also passes the fp64 oracle."""
    import torch
    from oracle import ref
    from paper_2403_16863_amd import gemm as G, gemm_search as GS, inputs as I, sip
    from tests.test_gpu_gemm import check
    variant = G.gemm_lrelu_default_variant(I.GEMM_M, I.GEMM_N, I.GEMM_K)
    d = tempfile.mkdtemp(prefix="sip_gemm_gpu_")
    try:
        k = sip.Kernel(sip.compile_gemm_base(d, I.F16, G.gemm_lrelu_variant_knobs(variant)), loop_depth=1)
        run = sip.GemmRunner(k, variant, I.F16, d, samples=6, seed=1)
        x0 = sip.Schedule(tuple(k.nodes))
        assert run.admit(x0)                                   # bit-identical on six shapes
        h = run.handle(x0)
        a = torch.zeros((32, 64), dtype=torch.bfloat16, device="cuda")
        with pytest.raises(G.GemmError):                       # loaded for binary16
            G.gemm_lrelu_codeobj(h, a, a.t().contiguous(), torch.zeros((32, 32), dtype=torch.bfloat16, device="cuda"), 0.1)
        with pytest.raises(G.GemmError):
            G.gemm_lrelu_codeobj_load("/nonexistent.co", k.name, variant, I.F16)
    finally:
        shutil.rmtree(d, ignore_errors=True)
    res = sip.search_gemm(seed=2, cool=1.25, samples=6, validate_rounds=2, keep_best=None)
    assert res["steps"] >= 15 and res["admitted"] >= 1 and res["movable_instructions"] >= 10
    assert res["best_us"] <= res["unmodified_codeobj_us"]
    # the winner's assembly, reloaded, against the oracle on a ragged shape
    d = tempfile.mkdtemp(prefix="sip_gemm_gpu_")
    try:
        best_s = d + "/best.s"
        res = sip.search_gemm(seed=2, cool=1.25, samples=6, validate_rounds=1, keep_best=best_s)
        text = open(best_s).read()
        name = sip.Kernel(text, loop_depth=1).name
        h = G.gemm_lrelu_codeobj_load(sip.assemble(text, d, "best"), name, variant, I.F16)
        for (M, N, K) in ((100, 72, 328), (I.GEMM_M, I.GEMM_N, I.GEMM_K)):
            ab, bb = I.make_gemm(M, N, K, I.F16, seed=8)
            a, b = GS._device(ab, I.F16), GS._device(bb, I.F16)
            c = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
            G.gemm_lrelu_codeobj(h, a, b, c, I.GEMM_SLOPE)
            torch.cuda.synchronize()
            check(c.to(torch.float64).cpu().numpy(), ab, bb, I.GEMM_SLOPE, I.F16, f"searched kernel M{M} N{N} K{K}")
        G.gemm_lrelu_codeobj_unload(h)
    finally:
        shutil.rmtree(d, ignore_errors=True)
