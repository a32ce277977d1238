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
        out = sip.search_workload(2, seed=3, t_max=0.05, t_min=0.025, cool=1.05, samples=8, keep_best=d + "/best.s")
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
    finally:
        shutil.rmtree(d, ignore_errors=True)
