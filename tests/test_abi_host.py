"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol
the header declares, describes its variant lattice consistently and rejects bad
arguments before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2403_16863_amd as A
from paper_2403_16863_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(attn_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    L = binding.lib()
    names = declared_symbols()
    assert len(names) >= 10
    for n in names:
        assert hasattr(L, n), f"libattn.so does not export {n}"
        assert hasattr(binding, n), f"binding has no function {n}"
    assert sorted(binding.SYMBOLS) == names


def test_variant_table_is_consistent():
    nv = A.attn_num_variants()
    assert nv >= 1
    nk = A.attn_num_knobs()
    sizes = [A.attn_knob_size(k) for k in range(nk)]
    assert all(A.attn_knob_name(k) for k in range(nk))
    seen = set()
    for v in range(nv):
        c = A.attn_variant_coords(v)
        assert len(c) == nk and all(0 <= ci < si for ci, si in zip(c, sizes))
        assert c not in seen
        seen.add(c)
        assert A.attn_variant_from_coords(c) == v
        assert "bn=" in A.attn_variant_desc(v)
    assert A.attn_variant_from_coords([s - 1 for s in sizes]) in (None, *range(nv))
    for d in (64, 128):
        for dt in (0, 1):
            for causal in (False, True):
                dv = A.attn_default_variant(4096, d, dt, causal)
                assert A.attn_variant_supported(dv, d, dt, causal)
    with pytest.raises(A.AttnError):
        A.attn_variant_desc(nv)
    with pytest.raises(A.AttnError):
        A.attn_variant_coords(-1)
    assert binding.strerror(0) == "ok" and "invalid" in binding.strerror(-1)


def test_bad_arguments_are_rejected_on_the_host():
    """check happens before any launch, so fake (never dereferenced) pointers do."""
    L = binding.lib()
    p = lambda x: ctypes.c_void_p(x)
    good = dict(q=0x10000, k=0x20000, v=0x30000, out=0x40000, lse=0x50000)

    def call(B=1, H=1, N=16, d=64, causal=0, scale=1.0, dtype=0, **over):
        a = dict(good, **over)
        return L.attn_fwd(p(a["q"]), p(a["k"]), p(a["v"]), p(a["out"]), p(a["lse"]),
                          B, H, N, d, causal, scale, dtype, None)

    assert call(q=0) == binding.ATTN_EINVAL
    assert call(lse=0) == binding.ATTN_EINVAL
    assert call(N=0) == binding.ATTN_EINVAL
    assert call(B=-1) == binding.ATTN_EINVAL
    assert call(dtype=2) == binding.ATTN_EINVAL
    assert call(scale=float("inf")) == binding.ATTN_EINVAL
    assert call(k=0x20008) == binding.ATTN_EINVAL            # misaligned
    assert call(out=0x10000 + 64) == binding.ATTN_EINVAL     # out overlaps q
    assert call(lse=0x40000) == binding.ATTN_EINVAL          # lse overlaps out
    assert call(d=32) == binding.ATTN_EUNSUPPORTED
    assert call(d=256) == binding.ATTN_EUNSUPPORTED
    ms = (ctypes.c_float * 1)()
    assert L.attn_time_variant(p(1 << 16), p(2 << 16), p(3 << 16), p(4 << 16), p(5 << 16),
                               1, 1, 16, 64, 0, 1.0, 0, None, 0, 0, 0, ms) == binding.ATTN_EINVAL
