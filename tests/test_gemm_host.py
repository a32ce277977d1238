"""Host-side checks of the GEMM + LeakyReLU boundary that need no GPU: the library exports every
symbol include/gemm_lrelu.h declares, the block -> tile map covers every tile once and keeps
an XCD's tiles compact, and bad arguments are rejected before any launch."""
import ctypes
import os
import re

import pytest

from paper_2403_16863_amd import gemm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported_and_bound():
    text = open(os.path.join(ROOT, "include", "gemm_lrelu.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(gemm_lrelu[a-z_0-9]*)\s*\(", text)))
    L = gemm.lib()
    assert len(names) == 11
    for n in names:
        assert hasattr(L, n), f"libattn.so does not export {n}"
        assert hasattr(gemm, n), f"binding has no function {n}"
    assert sorted(gemm.SYMBOLS) == names


@pytest.mark.parametrize("ntm,ntn", [(16, 16), (1, 1), (1, 7), (3, 5), (7, 9), (16, 17), (5, 64), (33, 3)])
def test_tile_map_is_a_bijection(ntm, ntn):
    seen = set()
    for b in range(ntm * ntn):
        tm, tn = gemm.gemm_lrelu_tile_of_block(b, ntm, ntn)
        assert 0 <= tm < ntm and 0 <= tn < ntn
        seen.add((tm, tn))
    assert len(seen) == ntm * ntn
    for bad in (-1, ntm * ntn):
        with pytest.raises(gemm.GemmError):
            gemm.gemm_lrelu_tile_of_block(bad, ntm, ntn)


def test_tile_map_keeps_an_xcd_compact_on_the_paper_shape():
    """512 x 512: 16 x 16 tiles, 32 per XCD (workgroup b runs on XCD b % 8): each XCD's tiles
    touch 4 row strips of A and 8 column strips of B, not all 16 of either."""
    for x in range(8):
        tiles = [gemm.gemm_lrelu_tile_of_block(b, 16, 16) for b in range(x, 256, 8)]
        assert len({t[0] for t in tiles}) == 4
        assert len({t[1] for t in tiles}) == 8


def test_variant_table():
    nv = gemm.gemm_lrelu_num_variants()
    assert nv >= 4
    seen = set()
    for v in range(nv):
        wk, bkw, stages, rot = gemm.gemm_lrelu_variant_knobs(v)
        assert wk in (1, 2, 4, 8) and bkw in (32, 64) and stages >= 3
        assert wk * stages * bkw * 128 <= 160 * 1024        # LDS of one workgroup
        assert rot in (0, 1) and (wk, bkw, stages, rot) not in seen
        seen.add((wk, bkw, stages, rot))
    assert 0 <= gemm.gemm_lrelu_default_variant(512, 512, 2048) < nv
    with pytest.raises(gemm.GemmError):
        gemm.gemm_lrelu_variant_knobs(nv)


def test_bad_arguments_are_rejected_on_the_host():
    """The check happens before any launch, so fake (never dereferenced) pointers do."""
    L = gemm.lib()
    p = ctypes.c_void_p

    def call(a=0x100000, b=0x200000, c=0x300000, M=32, N=32, K=32, dtype=0, variant=None):
        if variant is None:
            return L.gemm_lrelu(p(a), p(b), p(c), M, N, K, 0.01, dtype, None)
        return L.gemm_lrelu_variant(p(a), p(b), p(c), M, N, K, 0.01, dtype, None, variant)

    E = gemm.GEMM_EINVAL
    assert call(a=0) == E and call(b=0) == E and call(c=0) == E
    assert call(a=0x100008) == E                  # misaligned
    assert call(M=0) == E and call(N=0) == E and call(K=0) == E
    assert call(N=36) == E and call(K=12) == E    # rows must start on 16-byte boundaries
    assert call(N=1 << 24) == E and call(K=1 << 24) == E
    assert call(dtype=2) == E
    assert call(variant=-1) == E and call(variant=gemm.gemm_lrelu_num_variants()) == E
    assert call(c=0x100000 + 64) == E             # C overlaps A
    assert call(c=0x200000 - 16) == E             # C runs into B
    ms = ctypes.c_float()
    assert L.gemm_lrelu_time(p(0x100000), p(0x200000), p(0x300000), 32, 32, 32, 0.01, 0, None, 0, 0, 0,
                             ctypes.byref(ms)) == E
