"""Helpers shared by the GPU parity tests: run the HIP path through the C-ABI
binding on uint16 bit patterns and compare with the CPU oracle."""
import numpy as np

from paper_2403_16863_amd import inputs as I

# Tolerances from the build's target statement: max |dO| on unit-scale outputs and
# |d lse| <= 1e-3 * max(1, |lse|).
O_TOL = {I.F16: 1e-2, I.BF16: 3e-2}
LSE_RTOL = 1e-3
# Half-unit roundoff of the 16-bit types.  For inputs beyond unit scale the error of O is bounded
# relative to the largest |V|: u * sum_j p_j |v_j| from rounding P to 16 bits, u * |O| from the
# final rounding, fp32 terms far below both, i.e. at most about 2 u max|V|.  The absolute
# tolerances above are that bound at max|V| = 10 (binary16) and 3.8 (bfloat16).
U = {I.F16: 2.0 ** -11, I.BF16: 2.0 ** -8}


def o_tol(dtype, vmax):
    """Tolerance on max |dO| for inputs whose largest |V| is vmax: the absolute one of the target
    statement up to the V magnitude where the error bound reaches it, the bound beyond."""
    return max(O_TOL[dtype], 2.1 * U[dtype] * float(vmax))


def torch_dtype(dtype):
    import torch
    return torch.float16 if dtype == I.F16 else torch.bfloat16


def to_device(bits, dtype):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to("cuda")
    return t.view(torch_dtype(dtype))


def run_gpu(qb, kb, vb, causal, scale, dtype, variant=None, poison=True):
    """Returns (O float64 [B,H,N,d], lse float64 [B,H,N]) from the HIP path."""
    import torch
    import paper_2403_16863_amd as A
    q, k, v = (to_device(a, dtype) for a in (qb, kb, vb))
    out = torch.empty_like(q)
    lse = torch.empty(q.shape[:3], dtype=torch.float32, device="cuda")
    if poison:  # every output element must be overwritten
        out.fill_(float("nan"))
        lse.fill_(float("nan"))
    if variant is None:
        A.attn_fwd(q, k, v, out, lse, causal, scale)
    else:
        A.attn_fwd_variant(q, k, v, out, lse, causal, scale, variant)
    torch.cuda.synchronize()
    return out.to(torch.float64).cpu().numpy(), lse.to(torch.float64).cpu().numpy()


def check(O_gpu, lse_gpu, O_ref, lse_ref, dtype, out_scale=1.0, what=""):
    assert np.isfinite(O_gpu).all(), f"{what}: non-finite O"
    assert np.isfinite(lse_gpu).all(), f"{what}: non-finite lse"
    eo = float(np.max(np.abs(O_gpu - O_ref))) if O_ref.size else 0.0
    el = float(np.max(np.abs(lse_gpu - lse_ref) / np.maximum(1.0, np.abs(lse_ref)))) if lse_ref.size else 0.0
    assert eo <= O_TOL[dtype] * out_scale, f"{what}: max|dO| = {eo:.3e} > {O_TOL[dtype] * out_scale:.1e}"
    assert el <= LSE_RTOL, f"{what}: lse error {el:.3e} > {LSE_RTOL:.0e}"
    return eo, el
