"""Host logic of the strategy comparison and the knob attribution, on made-up timing tables."""
import random

from paper_2403_16863_amd import search_compare as SC


def model_table(noise=0.004, reps=9, seed=0):
    """Three knobs; the first one matters a lot, the second a little, the third not at all."""
    rng = random.Random(seed)
    table = {}
    for a in (1, 2, 4, 8):
        for b in (32, 64):
            for c in (3, 4, 8):
                if (a, b, c) in ((8, 64, 8), (1, 32, 3)):
                    continue                                  # holes, as in a real variant table
                t = 10.0 * {1: 1.8, 2: 1.3, 4: 1.0, 8: 1.02}[a] * {32: 1.0, 64: 0.97}[b]
                table[(a, b, c)] = [t * (1.0 + rng.gauss(0.0, noise)) for _ in range(reps)]
    return table


def test_every_strategy_respects_its_budget_and_is_reproducible():
    table = model_table()
    keys = sorted(table)
    for name in SC.STRATEGIES:
        for budget in (1, 3, 10, 60):
            calls = []
            rng = random.Random(5)

            def measure(k):
                calls.append(k)
                return rng.choice(table[k])
            pick, seen = SC.run_strategy(name, keys, keys[0], measure, budget, seed=7)
            assert len(calls) == budget, (name, budget)
            assert pick in table and seen <= min(budget, len(keys))
        one = [SC.run_strategy(name, keys, keys[0], lambda k: table[k][0], 15, seed=3) for _ in range(2)]
        assert one[0] == one[1]


def test_with_enough_budget_every_strategy_finds_a_best_variant():
    table = model_table()
    res = SC.compare(table, start=(1, 64, 8), budgets=(5, len(table), 4 * len(table)), seeds=20)
    for name, rows in res.items():
        assert rows[-1]["mean_regret"] < 0.01, name
        assert rows[-1]["mean_regret"] <= rows[0]["mean_regret"] + 1e-9, name
    assert res["exhaustive"][1]["within_half_percent"] >= 0.9      # one full sweep of a quiet table
    # five measurements cannot cover 22 variants: a neighbourhood search from a bad start still gets closer than a sweep in table order
    assert res["hill_climb"][0]["mean_regret"] < res["exhaustive"][0]["mean_regret"]


def test_attribution_ranks_the_knobs():
    att = SC.attribution(model_table(), ("a", "b", "c"))
    k = att["knobs"]
    assert att["r2_main_effects"] > 0.99
    assert k["a"]["spread_percent"] > 70 and 2 < k["b"]["spread_percent"] < 4 and k["c"]["spread_percent"] < 1
    assert k["a"]["fit_lost_without"] > 0.9 > k["b"]["fit_lost_without"] > k["c"]["fit_lost_without"]
    assert k["a"]["levels"] == [1, 2, 4, 8]
    assert abs(k["a"]["effect_percent"][2] - (100 * (1.0 / 1.8 - 1))) < 1.0      # level 4 against level 1
    assert k["b"]["one_knob_pairs"] == 10 and abs(k["b"]["mean_abs_change_percent"] - 100 * (1 / 0.97 - 1)) < 0.5


def test_measure_table_keeps_rejected_variants_out():
    keys = [(1, 1), (1, 2), (2, 1)]
    n = {"calls": 0}

    def measure(k):
        n["calls"] += 1
        return float(sum(k))
    table, rejected = SC.measure_table(keys, measure, lambda k: k != (1, 2), reps=3)
    assert rejected == [(1, 2)] and sorted(table) == [(1, 1), (2, 1)] and n["calls"] == 6
    assert table[(2, 1)] == [3.0, 3.0, 3.0]
