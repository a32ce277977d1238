"""Host-side tests of the work-item schedule (no GPU): the function the kernels call to pick
their items is exported through the C ABI and checked here as plain host logic."""
import itertools

import pytest

import paper_2403_16863_amd as A


def items_of(grid, BH, nqt):
    """{workgroup: [(bh, qt), ...]} by walking rounds until a workgroup runs dry."""
    out = {}
    for g in range(grid):
        seq = []
        for rnd in itertools.count():
            it = A.attn_schedule_item(grid, g, BH, nqt, rnd)
            if it is None:
                # once dry, always dry
                assert A.attn_schedule_item(grid, g, BH, nqt, rnd + 1) is None
                break
            seq.append(it)
        out[g] = seq
    return out


@pytest.mark.parametrize("grid,BH,nqt", [
    (256, 64, 16), (256, 32, 64), (512, 128, 16), (256, 64, 4), (8, 8, 1), (16, 8, 5),
    (7, 3, 5), (1, 1, 1), (1, 5, 7), (30, 6, 5), (256, 2, 1), (24, 40, 3), (256, 24, 11), (255, 64, 16),
])
def test_every_item_exactly_once(grid, BH, nqt):
    sched = items_of(grid, BH, nqt)
    seen = [it for seq in sched.values() for it in seq]
    assert len(seen) == BH * nqt
    assert set(seen) == {(b, q) for b in range(BH) for q in range(nqt)}


@pytest.mark.parametrize("grid,BH,nqt", [(256, 64, 16), (256, 32, 64), (512, 128, 16), (64, 16, 8)])
def test_heads_stay_on_their_xcd(grid, BH, nqt):
    # grid and BH multiples of 8: workgroup g runs on XCD g % 8 and only touches heads = g mod 8
    for g, seq in items_of(grid, BH, nqt).items():
        assert all(bh % 8 == g % 8 for bh, _ in seq)


@pytest.mark.parametrize("grid,BH,nqt", [(256, 64, 16), (256, 32, 64), (512, 128, 16), (256, 64, 8)])
def test_balanced_and_local(grid, BH, nqt):
    # causal weight of query tile qt is proportional to qt + 1
    sched = items_of(grid, BH, nqt)
    loads = [sum(qt + 1 for _, qt in seq) for seq in sched.values()]
    assert max(loads) - min(loads) <= 1 + nqt // 8   # serpentine deal: near-equal sums
    # in every round the workgroups of one XCD work on few heads (their K/V share that L2)
    per_xcd = grid // 8
    rounds = max(len(seq) for seq in sched.values())
    for x in range(8):
        for rnd in range(rounds):
            heads = {sched[g][rnd][0] for g in range(x, grid, 8) if rnd < len(sched[g])}
            assert len(heads) <= -(-per_xcd // nqt) + 1


def test_grid_size():
    v = A.attn_default_variant(4096, 128, A.ATTN_BF16, True)
    assert A.attn_schedule_grid(v, 256, 2, 32, 4096) == 256           # one persistent workgroup per CU
    assert A.attn_schedule_grid(v, 256, 1, 2, 128) == 2               # never more than items
    assert A.attn_schedule_grid(v, 256, 1, 8, 256) == 8
    v64 = A.attn_default_variant(1024, 64, A.ATTN_F16, True)
    g = A.attn_schedule_grid(v64, 256, 4, 16, 1024)
    assert 0 < g <= 512 and g % 8 == 0
    with pytest.raises(A.AttnError):
        A.attn_schedule_grid(v, 0, 1, 1, 1)
    with pytest.raises(A.AttnError):
        A.attn_schedule_item(4, 4, 1, 1, 0)
