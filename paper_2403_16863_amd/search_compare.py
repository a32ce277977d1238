"""Search strategies compared on one schedule space, and attribution of the gain to knobs.

The paper searches with simulated annealing (Alg. 1) and names better search methods and the
question "which change is it that helps" as future work (Sec. 5.3 end, Sec. 6).  The variant
tables of this library are small enough to measure completely, which gives a ground truth to
score strategies against:

* `measure_table` times every admitted variant `reps` times, round-robin (so that slow drifts
  of the device hit all variants alike);
* the strategies (`STRATEGIES`: exhaustive sweep in table order, random search, simulated
  annealing - the loop of Alg. 1 itself -, first-improvement hill climbing, and a
  lower-confidence-bound bandit that can re-measure) are host logic over a noisy `measure(key)`;
  `compare` replays them against the table (one measurement = one draw from that variant's
  recorded timings) for several budgets and seeds and reports the regret
  t(chosen) / t(best) - 1 under the table's means;
* `attribution` fits log t = sum of per-knob level effects by least squares and lists, per
  knob, the spread of its fitted effects, the loss of fit when the knob is left out, and the
  observed changes between variants that differ in that knob only.

  python -m paper_2403_16863_amd.search_compare --space gemm
  python -m paper_2403_16863_amd.search_compare --space attn --workload 2
"""
from __future__ import annotations

import argparse
import json
import math
import random
import statistics
from typing import Callable, Dict, List, Optional, Sequence, Tuple

from .search import anneal_states

Key = Tuple[int, ...]
Table = Dict[Key, List[float]]


def neighbours(keys: Sequence[Key], x: Key) -> List[Key]:
    """Variants that differ from x in exactly one knob."""
    return sorted(k for k in keys if sum(a != b for a, b in zip(k, x)) == 1)


class _Budget(Exception):
    pass


class Meter:
    """Counts measurements, remembers them, and stops a strategy when the budget is spent."""

    def __init__(self, measure: Callable[[Key], float], budget: int):
        self.measure, self.budget, self.seen = measure, budget, {}

    def __call__(self, key: Key) -> float:
        if self.budget <= 0:
            raise _Budget()
        self.budget -= 1
        t = float(self.measure(key))
        self.seen.setdefault(key, []).append(t)
        return t

    def best(self) -> Optional[Key]:
        """Greedy ranking of everything stored (Sec. 4.1): the lowest mean measured time."""
        if not self.seen:
            return None
        return min(sorted(self.seen), key=lambda k: statistics.fmean(self.seen[k]))


def exhaustive(keys: Sequence[Key], start: Key, meter: Meter, rng: random.Random) -> None:
    while True:                                  # sweep after sweep until the budget ends
        for k in sorted(keys):
            meter(k)


def random_search(keys: Sequence[Key], start: Key, meter: Meter, rng: random.Random) -> None:
    meter(start)
    while True:
        order = sorted(keys)
        rng.shuffle(order)
        for k in order:
            meter(k)


def annealing(keys: Sequence[Key], start: Key, meter: Meter, rng: random.Random) -> None:
    def propose(x, r):
        near = neighbours(keys, x) or [k for k in sorted(keys) if k != x]
        return r.choice(near) if near else None
    while True:                                  # restart from the start point if the schedule cools down early
        anneal_states(start, propose, meter, lambda x: True, seed=rng.randrange(1 << 30), remeasure=False)
        if len(meter.seen) == len(keys):         # nothing new left to pay for: spend the rest re-measuring the leader
            while True:
                meter(meter.best())


def hill_climb(keys: Sequence[Key], start: Key, meter: Meter, rng: random.Random) -> None:
    x, t_x = start, meter(start)
    tried = {start}
    while True:
        near = [k for k in neighbours(keys, x) if k not in tried]
        if not near:                             # local optimum: jump to something unseen, or re-measure
            rest = [k for k in sorted(keys) if k not in tried]
            if not rest:
                while True:
                    meter(meter.best())
            near = [rng.choice(rest)]
        k = rng.choice(near)
        tried.add(k)
        t = meter(k)
        if t < t_x:
            x, t_x = k, t


def bandit(keys: Sequence[Key], start: Key, meter: Meter, rng: random.Random, c: float = 1.0) -> None:
    """Every arm once (random order, start first), then always the arm with the lowest
    mean - c * s * sqrt(2 ln n / n_arm), s = pooled standard deviation of repeated measurements
    (1 % of the mean until there are repeats)."""
    order = [k for k in sorted(keys) if k != start]
    rng.shuffle(order)
    for k in [start] + order:
        meter(k)
    n = len(keys)
    while True:
        n += 1
        devs = [t - statistics.fmean(v) for v in meter.seen.values() if len(v) > 1 for t in v]
        lead = statistics.fmean(meter.seen[meter.best()])
        s = math.sqrt(sum(d * d for d in devs) / len(devs)) if len(devs) > 1 else 0.01 * lead
        meter(min(sorted(meter.seen), key=lambda k: statistics.fmean(meter.seen[k])
                  - c * s * math.sqrt(2 * math.log(n) / len(meter.seen[k]))))


STRATEGIES: Dict[str, Callable] = {"exhaustive": exhaustive, "random": random_search, "annealing": annealing,
                                   "hill_climb": hill_climb, "bandit": bandit}


def run_strategy(name: str, keys: Sequence[Key], start: Key, measure: Callable[[Key], float], budget: int,
                 seed: int) -> Tuple[Key, int]:
    """The variant the strategy settles on after `budget` measurements, and how many variants it looked at."""
    meter = Meter(measure, budget)
    try:
        STRATEGIES[name](keys, start, meter, random.Random(seed))
    except _Budget:
        pass
    return meter.best(), len(meter.seen)


def compare(table: Table, start: Key, budgets: Sequence[int], seeds: int = 50) -> dict:
    """Replay every strategy against the measured table."""
    keys = sorted(table)
    truth = {k: statistics.fmean(v) for k, v in table.items()}
    t_best = min(truth.values())
    out = {}
    for name in STRATEGIES:
        rows = []
        for budget in budgets:
            regrets, hits = [], 0
            for seed in range(seeds):
                draw = random.Random(1000003 * seed + budget)
                pick, _ = run_strategy(name, keys, start, lambda k: draw.choice(table[k]), budget, seed)
                regrets.append(truth[pick] / t_best - 1.0)
                hits += truth[pick] <= t_best * 1.005
            rows.append({"budget": budget, "mean_regret": statistics.fmean(regrets), "max_regret": max(regrets),
                         "within_half_percent": hits / seeds})
        out[name] = rows
    return out


def attribution(table: Table, knob_names: Sequence[str]) -> dict:
    """Which knob matters: least-squares main effects on log time, and one-knob contrasts."""
    import numpy as np
    keys = sorted(table)
    y = np.log(np.array([statistics.fmean(table[k]) for k in keys]))
    levels = [sorted({k[j] for k in keys}) for j in range(len(knob_names))]

    def design(skip: Optional[int]):
        cols = [np.ones(len(keys))]
        for j, lv in enumerate(levels):
            if j == skip:
                continue
            for v in lv[1:]:
                cols.append(np.array([1.0 if k[j] == v else 0.0 for k in keys]))
        return np.stack(cols, axis=1)

    def fit(skip: Optional[int]):
        X = design(skip)
        beta, *_ = np.linalg.lstsq(X, y, rcond=None)
        res = y - X @ beta
        return beta, float(res @ res)

    ss_tot = float(((y - y.mean()) ** 2).sum())
    beta, ss_full = fit(None)
    knobs = {}
    pos = 1
    for j, name in enumerate(knob_names):
        eff = [0.0] + [float(b) for b in beta[pos:pos + len(levels[j]) - 1]]
        pos += len(levels[j]) - 1
        _, ss_without = fit(j)
        pairs = [(a, b) for a in keys for b in keys if a < b and all((x == z) == (i != j) for i, (x, z) in enumerate(zip(a, b)))]
        changes = [abs(math.log(statistics.fmean(table[a]) / statistics.fmean(table[b]))) for a, b in pairs]
        knobs[name] = {
            "levels": levels[j],
            "effect_percent": [100.0 * (math.exp(e) - 1.0) for e in eff],          # relative to the first level
            "spread_percent": 100.0 * (math.exp(max(eff) - min(eff)) - 1.0),
            "fit_lost_without": (ss_without - ss_full) / ss_tot if ss_tot > 0 else 0.0,
            "one_knob_pairs": len(pairs),
            "mean_abs_change_percent": 100.0 * (math.exp(statistics.fmean(changes)) - 1.0) if changes else None,
        }
    return {"r2_main_effects": 1.0 - ss_full / ss_tot if ss_tot > 0 else 1.0, "knobs": knobs}


def measure_table(keys: Sequence[Key], measure: Callable[[Key], float], admit: Callable[[Key], bool],
                  reps: int = 7, log: Optional[Callable[[str], None]] = None) -> Tuple[Table, List[Key]]:
    """Times every admitted key `reps` times, one round over all keys after the other."""
    rejected = [k for k in sorted(keys) if not admit(k)]
    table: Table = {k: [] for k in sorted(keys) if k not in rejected}
    for r in range(reps):
        for k in table:
            table[k].append(float(measure(k)))
        if log:
            log(f"round {r + 1} of {reps} done")
    return table, rejected


def gemm_space(dtype: int = 0):
    import torch
    from . import gemm, gemm_search as GS, inputs as I
    lib_table = GS.library_table()
    ab, bb = I.make_gemm(I.GEMM_M, I.GEMM_N, I.GEMM_K, dtype, 0)
    a, b = GS._device(ab, dtype), GS._device(bb, dtype)
    c = torch.empty((I.GEMM_M, I.GEMM_N), dtype=a.dtype, device="cuda")
    start = next(k for k, v in lib_table.items() if v == gemm.gemm_lrelu_default_variant(I.GEMM_M, I.GEMM_N, I.GEMM_K))
    return (f"gemm_lrelu M{I.GEMM_M} N{I.GEMM_N} K{I.GEMM_K}", gemm.KNOB_NAMES, sorted(lib_table), start,
            lambda k: GS.measure_variant((a, b, c), lib_table[k], iters=1000),
            lambda k: GS.admit_against_default(lib_table[k], dtype, samples=6), "us")


def attn_space(widx: int):
    import torch
    from . import binding as Bd, inputs as I, search as S
    w = I.WORKLOADS[widx]
    lat = S.Lattice.from_library(w.d, w.dtype, w.causal)
    q, k, v = S._device_inputs(w.B, w.H, w.N, w.d, w.dtype, 1234 + widx, w.qk_sigma)
    out = torch.empty_like(q)
    lse = torch.empty(q.shape[:3], dtype=torch.float32, device="cuda")
    names = tuple(Bd.attn_knob_name(i) for i in range(Bd.attn_num_knobs()))
    start = tuple(Bd.attn_variant_coords(Bd.attn_default_variant(w.N, w.d, w.dtype, w.causal)))
    return (w.label, names, sorted(lat.points), start,
            lambda c: S.measure_variant((q, k, v, out, lse), w.causal, w.scale, lat.points[c], iters=20),
            lambda c: S.admit_against_default(lat.points[c], w.d, w.dtype, w.causal, samples=7), "ms")


def main(argv: Optional[Sequence[str]] = None) -> None:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--space", choices=("gemm", "attn"), default="gemm")
    ap.add_argument("--workload", type=int, default=2, help="attention workload index (with --space attn)")
    ap.add_argument("--reps", type=int, default=7)
    ap.add_argument("--seeds", type=int, default=50)
    a = ap.parse_args(argv)
    label, names, keys, start, measure, admit, unit = gemm_space() if a.space == "gemm" else attn_space(a.workload)
    table, rejected = measure_table(keys, measure, admit, a.reps, log=lambda s: print(s, flush=True))
    n = len(table)
    budgets = sorted({max(2, n // 4), max(3, n // 2), n, 2 * n, 4 * n})
    truth = {k: statistics.fmean(v) for k, v in table.items()}
    noise = statistics.fmean(statistics.pstdev(v) / statistics.fmean(v) for v in table.values())
    print(json.dumps({
        "workload": label, "knobs": list(names), "unit": unit, "variants": n, "rejected": [list(k) for k in rejected],
        "start": list(start), "t_start": truth[start], "best": list(min(truth, key=truth.get)), "t_best": min(truth.values()),
        "noise_relative_std": noise,
        "table": [{"key": list(k), "mean": truth[k], "min": min(table[k]), "max": max(table[k])} for k in sorted(truth, key=truth.get)],
        "strategies": compare(table, start, budgets, a.seeds),
        "attribution": attribution(table, names),
    }))


if __name__ == "__main__":
    main()
