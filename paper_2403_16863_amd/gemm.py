"""Thin ctypes binding over the C ABI declared in include/gemm_lrelu.h (fused GEMM + LeakyReLU,
the paper's second workload, Sec. 5 / Table 3).

Argument marshalling only: the product runs in the HIP kernel of libattn.so.  There is no
fallback: if the library has not been built, loading it fails loudly.
"""
from __future__ import annotations

import ctypes

from . import binding

GEMM_F16, GEMM_BF16 = 0, 1
GEMM_OK, GEMM_EINVAL, GEMM_ELAUNCH = 0, -1, -2
KNOB_NAMES = ("wk", "bkw", "stages", "rot")

# every symbol include/gemm_lrelu.h declares
SYMBOLS = ("gemm_lrelu", "gemm_lrelu_variant", "gemm_lrelu_num_variants", "gemm_lrelu_default_variant",
           "gemm_lrelu_variant_knobs", "gemm_lrelu_time", "gemm_lrelu_tile_of_block", "gemm_lrelu_codeobj_load",
           "gemm_lrelu_codeobj_unload", "gemm_lrelu_codeobj", "gemm_lrelu_time_codeobj")

_ready = False


class GemmError(RuntimeError):
    def __init__(self, code: int, what: str):
        names = {GEMM_EINVAL: "invalid argument", GEMM_ELAUNCH: "the HIP runtime refused the call"}
        super().__init__(f"{what}: {names.get(code, 'unknown error')} (code {code})")
        self.code = code


def lib():
    global _ready
    L = binding.lib()
    if not _ready:
        vp, i, f = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
        common = [vp, vp, vp, i, i, i, f, i, vp]
        L.gemm_lrelu.restype = i
        L.gemm_lrelu.argtypes = common
        L.gemm_lrelu_variant.restype = i
        L.gemm_lrelu_variant.argtypes = common + [i]
        L.gemm_lrelu_time.restype = i
        L.gemm_lrelu_time.argtypes = common + [i, i, i, ctypes.POINTER(f)]
        L.gemm_lrelu_num_variants.restype = i
        L.gemm_lrelu_num_variants.argtypes = []
        L.gemm_lrelu_default_variant.restype = i
        L.gemm_lrelu_default_variant.argtypes = [i, i, i]
        L.gemm_lrelu_variant_knobs.restype = i
        L.gemm_lrelu_variant_knobs.argtypes = [i, ctypes.POINTER(i)]
        L.gemm_lrelu_tile_of_block.restype = i
        L.gemm_lrelu_tile_of_block.argtypes = [i, i, i, ctypes.POINTER(i), ctypes.POINTER(i)]
        L.gemm_lrelu_codeobj_load.restype = i
        L.gemm_lrelu_codeobj_load.argtypes = [ctypes.c_char_p, ctypes.c_char_p, i, i]
        L.gemm_lrelu_codeobj_unload.restype = i
        L.gemm_lrelu_codeobj_unload.argtypes = [i]
        L.gemm_lrelu_codeobj.restype = i
        L.gemm_lrelu_codeobj.argtypes = [i] + common
        L.gemm_lrelu_time_codeobj.restype = i
        L.gemm_lrelu_time_codeobj.argtypes = [i] + common + [i, i, ctypes.POINTER(f)]
        _ready = True
    return L


def _marshal(a, b, c, stream):
    import torch
    for name, t in (("a", a), ("b", b), ("c", c)):
        if not t.is_cuda:
            raise ValueError(f"{name} must live in device memory")
        if not t.is_contiguous():
            raise ValueError(f"{name} must be contiguous")
    if a.dim() != 2 or b.dim() != 2 or c.dim() != 2 or a.shape[1] != b.shape[0] or \
            tuple(c.shape) != (a.shape[0], b.shape[1]):
        raise ValueError("a must be [M,K], b [K,N] and c [M,N]")
    if b.dtype != a.dtype or c.dtype != a.dtype:
        raise ValueError("a, b, c must share one dtype")
    if a.dtype == torch.float16:
        dt = GEMM_F16
    elif a.dtype == torch.bfloat16:
        dt = GEMM_BF16
    else:
        raise TypeError(f"inputs must be float16 or bfloat16, got {a.dtype}")
    if stream is None:
        stream = torch.cuda.current_stream(a.device).cuda_stream
    M, K = a.shape
    return (a.data_ptr(), b.data_ptr(), c.data_ptr(), M, b.shape[1], K), dt, stream


def gemm_lrelu(a, b, c, slope: float, stream=None) -> None:
    """c <- leaky_relu(a @ b) for device tensors a [M,K], b [K,N], c [M,N]; asynchronous on `stream`
    (an integer hipStream_t; default: torch's current stream)."""
    args, dt, st = _marshal(a, b, c, stream)
    rc = lib().gemm_lrelu(*args, float(slope), dt, st)
    if rc != GEMM_OK:
        raise GemmError(rc, "gemm_lrelu")


def gemm_lrelu_variant(a, b, c, slope: float, variant_id: int, stream=None) -> None:
    args, dt, st = _marshal(a, b, c, stream)
    rc = lib().gemm_lrelu_variant(*args, float(slope), dt, st, int(variant_id))
    if rc != GEMM_OK:
        raise GemmError(rc, "gemm_lrelu_variant")


def gemm_lrelu_time(a, b, c, slope: float, variant_id: int, warmup: int = 5, iters: int = 100, stream=None) -> float:
    """Milliseconds for `iters` launches issued back to back (one pair of events around all of them)."""
    args, dt, st = _marshal(a, b, c, stream)
    ms = ctypes.c_float(0.0)
    rc = lib().gemm_lrelu_time(*args, float(slope), dt, st, int(variant_id), int(warmup), int(iters), ctypes.byref(ms))
    if rc != GEMM_OK:
        raise GemmError(rc, "gemm_lrelu_time")
    return float(ms.value)


def gemm_lrelu_num_variants() -> int:
    return int(lib().gemm_lrelu_num_variants())


def gemm_lrelu_default_variant(M: int, N: int, K: int) -> int:
    return int(lib().gemm_lrelu_default_variant(int(M), int(N), int(K)))


def gemm_lrelu_variant_knobs(variant_id: int):
    """(wk, bkw, stages, rot) of a variant."""
    buf = (ctypes.c_int * 4)()
    rc = lib().gemm_lrelu_variant_knobs(int(variant_id), buf)
    if rc != GEMM_OK:
        raise GemmError(rc, "gemm_lrelu_variant_knobs")
    return tuple(buf)


def gemm_lrelu_tile_of_block(block: int, ntm: int, ntn: int):
    """(tm, tn): the 32 x 32 tile of C that workgroup `block` computes."""
    tm, tn = ctypes.c_int(0), ctypes.c_int(0)
    rc = lib().gemm_lrelu_tile_of_block(int(block), int(ntm), int(ntn), ctypes.byref(tm), ctypes.byref(tn))
    if rc != GEMM_OK:
        raise GemmError(rc, "gemm_lrelu_tile_of_block")
    return tm.value, tn.value


def gemm_lrelu_codeobj_load(path: str, kernel_name: str, variant_id: int, dtype: int) -> int:
    """Handle of a kernel loaded from a gfx950 code object, standing in for variant `variant_id`."""
    h = lib().gemm_lrelu_codeobj_load(path.encode(), kernel_name.encode(), int(variant_id), int(dtype))
    if h < 0:
        raise GemmError(h, "gemm_lrelu_codeobj_load")
    return h


def gemm_lrelu_codeobj_unload(handle: int) -> None:
    rc = lib().gemm_lrelu_codeobj_unload(int(handle))
    if rc != GEMM_OK:
        raise GemmError(rc, "gemm_lrelu_codeobj_unload")


def gemm_lrelu_codeobj(handle: int, a, b, c, slope: float, stream=None) -> None:
    args, dt, st = _marshal(a, b, c, stream)
    rc = lib().gemm_lrelu_codeobj(int(handle), *args, float(slope), dt, st)
    if rc != GEMM_OK:
        raise GemmError(rc, "gemm_lrelu_codeobj")


def gemm_lrelu_time_codeobj(handle: int, a, b, c, slope: float, warmup: int = 5, iters: int = 100, stream=None) -> float:
    args, dt, st = _marshal(a, b, c, stream)
    ms = ctypes.c_float(0.0)
    rc = lib().gemm_lrelu_time_codeobj(int(handle), *args, float(slope), dt, st, int(warmup), int(iters), ctypes.byref(ms))
    if rc != GEMM_OK:
        raise GemmError(rc, "gemm_lrelu_time_codeobj")
    return float(ms.value)
