"""Host logic of the GEMM schedule search: neighbourhoods on the variant table, and the annealing loop
driven by a made-up cost model (no GPU)."""
import random

from paper_2403_16863_amd import gemm, gemm_search as GS
from paper_2403_16863_amd.search import anneal_states


def test_neighbours_differ_in_one_knob_and_cover_the_table():
    table = GS.library_table()
    assert len(table) == gemm.gemm_lrelu_num_variants()
    for x in table:
        for y in GS.neighbours(table, x):
            assert sum(a != b for a, b in zip(x, y)) == 1 and y in table
    # every variant can be reached from the default by single-knob moves
    start = next(k for k, v in table.items() if v == gemm.gemm_lrelu_default_variant(512, 512, 2048))
    seen, todo = {start}, [start]
    while todo:
        for y in GS.neighbours(table, todo.pop()):
            if y not in seen:
                seen.add(y)
                todo.append(y)
    assert seen == set(table)


def test_search_finds_the_cheapest_admitted_variant_of_a_model():
    table = GS.library_table()
    cost = lambda x: 1.0 + 0.1 * abs(x[0] - 8) + 0.01 * abs(x[2] - 3) + 0.05 * x[3] + 0.001 * x[1]
    banned = min(table, key=cost)                      # the cheapest one fails its test
    want = min((k for k in table if k != banned), key=cost)
    start = max(table, key=cost)
    found = set()
    for seed in range(6):
        res = anneal_states(start, GS.propose_from(table), cost, lambda x: x != banned, seed=seed, cool=1.02)
        assert res.best != banned and banned not in res.times
        assert res.t_best <= res.t0
        found.add(res.best)
    assert want in found


def test_propose_is_reproducible():
    table = GS.library_table()
    p = GS.propose_from(table)
    x = next(iter(sorted(table)))
    assert [p(x, random.Random(3)) for _ in range(3)] == [p(x, random.Random(3))] * 3
