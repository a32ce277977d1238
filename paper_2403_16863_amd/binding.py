"""Thin ctypes binding over the C ABI declared in include/attn.h.

Argument marshalling only: every step of the attention forward runs in the HIP
kernels of libattn.so.  There is no fallback: if the library has not been built the
import of a symbol fails loudly.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libattn.so")

ATTN_F16, ATTN_BF16 = 0, 1
ATTN_OK, ATTN_EINVAL, ATTN_EUNSUPPORTED, ATTN_ELAUNCH = 0, -1, -2, -3

# every symbol include/attn.h declares
SYMBOLS = ("attn_fwd", "attn_fwd_variant", "attn_num_variants", "attn_variant_supported",
           "attn_variant_desc", "attn_num_knobs", "attn_knob_name", "attn_knob_size",
           "attn_variant_coords", "attn_variant_from_coords", "attn_default_variant",
           "attn_time_variant", "attn_strerror", "attn_schedule_grid", "attn_schedule_item", "attn_mfma_ceiling",
           "attn_valu_ceiling", "attn_mix_ceiling",
           "attn_codeobj_load", "attn_codeobj_unload", "attn_fwd_codeobj", "attn_time_codeobj",
           "attn_deploy_variant", "attn_deploy_codeobj", "attn_deploy_clear", "attn_deployed")

_lib = None


class AttnError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {strerror(code)} (code {code})")
        self.code = code


def lib():
    """Load libattn.so (built by __graft_entry__.build()); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; "
                              "g.build()'` from the repository root")
        # PyTorch ships its own HIP runtime under the same soname; load it first so
        # the library and torch's allocator/streams share ONE runtime instance.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i, f = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
        common = [vp, vp, vp, vp, vp, i, i, i, i, i, f, i, vp]
        L.attn_fwd.restype = i
        L.attn_fwd.argtypes = common
        L.attn_fwd_variant.restype = i
        L.attn_fwd_variant.argtypes = common + [i]
        L.attn_time_variant.restype = i
        L.attn_time_variant.argtypes = common + [i, i, i, ctypes.POINTER(ctypes.c_float)]
        L.attn_num_variants.restype = i
        L.attn_num_variants.argtypes = []
        L.attn_variant_supported.restype = i
        L.attn_variant_supported.argtypes = [i, i, i, i]
        L.attn_variant_desc.restype = i
        L.attn_variant_desc.argtypes = [i, ctypes.c_char_p, i]
        L.attn_num_knobs.restype = i
        L.attn_num_knobs.argtypes = []
        L.attn_knob_name.restype = ctypes.c_char_p
        L.attn_knob_name.argtypes = [i]
        L.attn_knob_size.restype = i
        L.attn_knob_size.argtypes = [i]
        L.attn_variant_coords.restype = i
        L.attn_variant_coords.argtypes = [i, ctypes.POINTER(i)]
        L.attn_variant_from_coords.restype = i
        L.attn_variant_from_coords.argtypes = [ctypes.POINTER(i)]
        L.attn_default_variant.restype = i
        L.attn_default_variant.argtypes = [i, i, i, i]
        L.attn_schedule_grid.restype = i
        L.attn_schedule_grid.argtypes = [i, i, i, i, i]
        L.attn_schedule_item.restype = i
        L.attn_schedule_item.argtypes = [i, i, i, i, i, ctypes.POINTER(i), ctypes.POINTER(i)]
        L.attn_codeobj_load.restype = i
        L.attn_codeobj_load.argtypes = [ctypes.c_char_p, ctypes.c_char_p, i, i, i, i]
        L.attn_codeobj_unload.restype = i
        L.attn_codeobj_unload.argtypes = [i]
        L.attn_deploy_variant.restype = i
        L.attn_deploy_variant.argtypes = [i, i, i, i, i, i]
        L.attn_deploy_codeobj.restype = i
        L.attn_deploy_codeobj.argtypes = [i, i, i]
        L.attn_deploy_clear.restype = i
        L.attn_deploy_clear.argtypes = []
        L.attn_deployed.restype = i
        L.attn_deployed.argtypes = [i, i, i, i, ctypes.POINTER(i), ctypes.POINTER(i)]
        L.attn_fwd_codeobj.restype = i
        L.attn_fwd_codeobj.argtypes = [i] + common
        L.attn_time_codeobj.restype = i
        L.attn_time_codeobj.argtypes = [i] + common + [i, i, ctypes.POINTER(ctypes.c_float)]
        L.attn_mfma_ceiling.restype = i
        L.attn_mfma_ceiling.argtypes = [i, i, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        L.attn_mix_ceiling.restype = i
        L.attn_mix_ceiling.argtypes = [i, i, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        L.attn_valu_ceiling.restype = i
        L.attn_valu_ceiling.argtypes = [i, i, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        L.attn_strerror.restype = ctypes.c_char_p
        L.attn_strerror.argtypes = [i]
        _lib = L
    return _lib


def attn_strerror(code: int) -> str:
    return lib().attn_strerror(int(code)).decode()


strerror = attn_strerror


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float16:
        return ATTN_F16
    if t.dtype == torch.bfloat16:
        return ATTN_BF16
    raise TypeError(f"attention inputs must be float16 or bfloat16, got {t.dtype}")


def _marshal(q, k, v, out, lse, stream):
    import torch
    for name, t in (("q", q), ("k", k), ("v", v), ("out", out), ("lse", lse)):
        if not t.is_cuda:
            raise ValueError(f"{name} must live in device memory")
        if not t.is_contiguous():
            raise ValueError(f"{name} must be contiguous")
    if q.dim() != 4 or k.shape != q.shape or v.shape != q.shape or out.shape != q.shape:
        raise ValueError("q, k, v, out must share one [B,H,N,d] shape")
    if k.dtype != q.dtype or v.dtype != q.dtype or out.dtype != q.dtype:
        raise ValueError("q, k, v, out must share one dtype")
    if lse.dtype != torch.float32 or tuple(lse.shape) != tuple(q.shape[:3]):
        raise ValueError("lse must be float32 [B,H,N]")
    B, H, N, d = q.shape
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    return (q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(),
            B, H, N, d), _dtype_code(q), stream


def attn_fwd(q, k, v, out, lse, causal: bool, scale: float, stream=None) -> None:
    """out, lse <- fused attention forward of device tensors q, k, v ([B,H,N,d]).
    Asynchronous on `stream` (an integer hipStream_t; default: torch's current stream)."""
    (ptrs_shape), dt, st = _marshal(q, k, v, out, lse, stream)
    rc = lib().attn_fwd(*ptrs_shape, int(bool(causal)), float(scale), dt, st)
    if rc != ATTN_OK:
        raise AttnError(rc, "attn_fwd")


def attn_fwd_variant(q, k, v, out, lse, causal: bool, scale: float, variant_id: int, stream=None) -> None:
    (ptrs_shape), dt, st = _marshal(q, k, v, out, lse, stream)
    rc = lib().attn_fwd_variant(*ptrs_shape, int(bool(causal)), float(scale), dt, st, int(variant_id))
    if rc != ATTN_OK:
        raise AttnError(rc, f"attn_fwd_variant({variant_id})")


def attn_time_variant(q, k, v, out, lse, causal: bool, scale: float, variant_id: int,
                      warmup: int = 10, iters: int = 50, stream=None):
    """Per-launch elapsed milliseconds (list of `iters` floats), HIP-event timed."""
    (ptrs_shape), dt, st = _marshal(q, k, v, out, lse, stream)
    ms = (ctypes.c_float * int(iters))()
    rc = lib().attn_time_variant(*ptrs_shape, int(bool(causal)), float(scale), dt, st,
                                 int(variant_id), int(warmup), int(iters), ms)
    if rc != ATTN_OK:
        raise AttnError(rc, f"attn_time_variant({variant_id})")
    return list(ms)


def attn_codeobj_load(path: str, kernel_name: str, variant_id: int, d: int, dtype: int, causal: bool) -> int:
    """Handle of a kernel loaded from a code object file (a re-scheduled copy of the kernel
    variant_id uses for this d, dtype, causal)."""
    rc = lib().attn_codeobj_load(os.fsencode(path), kernel_name.encode(), int(variant_id), int(d),
                                 int(dtype), int(bool(causal)))
    if rc < 0:
        raise AttnError(rc, f"attn_codeobj_load({path})")
    return rc


def attn_codeobj_unload(handle: int) -> None:
    rc = lib().attn_codeobj_unload(int(handle))
    if rc != ATTN_OK:
        raise AttnError(rc, "attn_codeobj_unload")


def attn_deploy_variant(variant_id: int, d: int, dtype: int, causal: bool, n_min: int = 1, n_max: int = 2 ** 31 - 1) -> None:
    """From now on attn_fwd launches this schedule for (d, dtype, causal) and n_min <= N <= n_max."""
    rc = lib().attn_deploy_variant(int(variant_id), int(d), int(dtype), int(bool(causal)), int(n_min), int(n_max))
    if rc != ATTN_OK:
        raise AttnError(rc, f"attn_deploy_variant({variant_id})")


def attn_deploy_codeobj(handle: int, n_min: int = 1, n_max: int = 2 ** 31 - 1) -> None:
    """From now on attn_fwd launches this loaded kernel for the shape class it was loaded for."""
    rc = lib().attn_deploy_codeobj(int(handle), int(n_min), int(n_max))
    if rc != ATTN_OK:
        raise AttnError(rc, f"attn_deploy_codeobj({handle})")


def attn_deploy_clear() -> None:
    rc = lib().attn_deploy_clear()
    if rc != ATTN_OK:
        raise AttnError(rc, "attn_deploy_clear")


def attn_deployed(N: int, d: int, dtype: int, causal: bool):
    """(matched, variant_id, handle): what attn_fwd launches for this shape; handle is -1
    unless a deployed code object matches, matched is False when the library default applies."""
    v, h = ctypes.c_int(-1), ctypes.c_int(-1)
    rc = lib().attn_deployed(int(N), int(d), int(dtype), int(bool(causal)), ctypes.byref(v), ctypes.byref(h))
    if rc < 0:
        raise AttnError(rc, "attn_deployed")
    return bool(rc), v.value, h.value


def attn_fwd_codeobj(handle: int, q, k, v, out, lse, causal: bool, scale: float, stream=None) -> None:
    (ptrs_shape), dt, st = _marshal(q, k, v, out, lse, stream)
    rc = lib().attn_fwd_codeobj(int(handle), *ptrs_shape, int(bool(causal)), float(scale), dt, st)
    if rc != ATTN_OK:
        raise AttnError(rc, f"attn_fwd_codeobj({handle})")


def attn_time_codeobj(handle: int, q, k, v, out, lse, causal: bool, scale: float,
                      warmup: int = 10, iters: int = 50, stream=None):
    """Per-launch elapsed milliseconds of a loaded kernel, HIP-event timed."""
    (ptrs_shape), dt, st = _marshal(q, k, v, out, lse, stream)
    ms = (ctypes.c_float * int(iters))()
    rc = lib().attn_time_codeobj(int(handle), *ptrs_shape, int(bool(causal)), float(scale), dt, st,
                                 int(warmup), int(iters), ms)
    if rc != ATTN_OK:
        raise AttnError(rc, f"attn_time_codeobj({handle})")
    return list(ms)


def attn_num_variants() -> int:
    return lib().attn_num_variants()


def attn_variant_supported(variant_id: int, d: int, dtype: int, causal: bool) -> bool:
    rc = lib().attn_variant_supported(int(variant_id), int(d), int(dtype), int(bool(causal)))
    if rc < 0:
        raise AttnError(rc, "attn_variant_supported")
    return bool(rc)


def attn_variant_desc(variant_id: int) -> str:
    buf = ctypes.create_string_buffer(256)
    rc = lib().attn_variant_desc(int(variant_id), buf, len(buf))
    if rc < 0:
        raise AttnError(rc, "attn_variant_desc")
    return buf.value.decode()


def attn_num_knobs() -> int:
    return lib().attn_num_knobs()


def attn_knob_name(knob: int) -> str:
    s = lib().attn_knob_name(int(knob))
    if s is None:
        raise AttnError(ATTN_EINVAL, "attn_knob_name")
    return s.decode()


def attn_knob_size(knob: int) -> int:
    rc = lib().attn_knob_size(int(knob))
    if rc < 0:
        raise AttnError(rc, "attn_knob_size")
    return rc


def attn_variant_coords(variant_id: int):
    n = attn_num_knobs()
    arr = (ctypes.c_int * n)()
    rc = lib().attn_variant_coords(int(variant_id), arr)
    if rc != ATTN_OK:
        raise AttnError(rc, "attn_variant_coords")
    return tuple(arr)


def attn_variant_from_coords(coords):
    """Variant id at a lattice point, or None if nothing is built there."""
    n = attn_num_knobs()
    if len(coords) != n:
        raise ValueError(f"need {n} coordinates")
    arr = (ctypes.c_int * n)(*[int(c) for c in coords])
    rc = lib().attn_variant_from_coords(arr)
    return None if rc < 0 else rc


def attn_schedule_grid(variant: int, compute_units: int, B: int, H: int, N: int) -> int:
    """Grid size (persistent workgroups) a launch of this variant uses."""
    rc = lib().attn_schedule_grid(int(variant), int(compute_units), int(B), int(H), int(N))
    if rc < 0:
        raise AttnError(rc, "attn_schedule_grid")
    return rc


def attn_schedule_item(grid: int, workgroup: int, BH: int, nqt: int, rnd: int):
    """(bh, qt) of the item a workgroup takes in a round, or None when it has none."""
    bh, qt = ctypes.c_int(0), ctypes.c_int(0)
    rc = lib().attn_schedule_item(int(grid), int(workgroup), int(BH), int(nqt), int(rnd),
                                  ctypes.byref(bh), ctypes.byref(qt))
    if rc < 0:
        raise AttnError(rc, "attn_schedule_item")
    return (bh.value, qt.value) if rc == 1 else None


def attn_mfma_ceiling(random_operands: bool, iters: int = 300000):
    """(TFLOP/s, core clock in GHz) of a kernel of back-to-back bf16 MFMAs; see the header."""
    import torch
    counters = torch.zeros(3, dtype=torch.int64, device="cuda")
    tf, ghz = ctypes.c_double(0), ctypes.c_double(0)
    rc = lib().attn_mfma_ceiling(int(bool(random_operands)), int(iters), torch.cuda.current_stream().cuda_stream, counters.data_ptr(),
                                 ctypes.byref(tf), ctypes.byref(ghz))
    if rc != 0:
        raise AttnError(rc, "attn_mfma_ceiling")
    return tf.value, ghz.value


def attn_mix_ceiling(mode: int, iters: int = 150000):
    """(TFLOP/s, core clock in GHz) of the tile loop's own instruction mix; see the header."""
    import torch
    counters = torch.zeros(3, dtype=torch.int64, device="cuda")
    tf, ghz = ctypes.c_double(0), ctypes.c_double(0)
    rc = lib().attn_mix_ceiling(int(mode), int(iters), torch.cuda.current_stream().cuda_stream, counters.data_ptr(),
                                ctypes.byref(tf), ctypes.byref(ghz))
    if rc != 0:
        raise AttnError(rc, "attn_mix_ceiling")
    return tf.value, ghz.value


def attn_valu_ceiling(waves_per_simd: int, iters: int = 200000):
    """(score elements per second, core clock in GHz) of the softmax's own instruction mix; see the header."""
    import torch
    counters = torch.zeros(3, dtype=torch.int64, device="cuda")
    eps, ghz = ctypes.c_double(0), ctypes.c_double(0)
    rc = lib().attn_valu_ceiling(int(waves_per_simd), int(iters), torch.cuda.current_stream().cuda_stream, counters.data_ptr(),
                                 ctypes.byref(eps), ctypes.byref(ghz))
    if rc != 0:
        raise AttnError(rc, "attn_valu_ceiling")
    return eps.value, ghz.value


def attn_default_variant(N: int, d: int, dtype: int, causal: bool) -> int:
    return lib().attn_default_variant(int(N), int(d), int(dtype), int(bool(causal)))
