"""Host-side tests of the annealing search (Alg. 1, Eq. 1, Sec. 3.2 mutation policy) on
synthetic energy landscapes; no GPU.  The paper fixes no hyper-parameters and prints no
trajectory, so the trajectory itself is unpinned: what is tested are the algorithm's
invariants and its special cases."""
import math
import random

import pytest

from paper_2403_16863_amd import search as S


def box(sizes, holes=()):
    pts, n = {}, 0
    def rec(prefix):
        nonlocal n
        if len(prefix) == len(sizes):
            if tuple(prefix) not in holes:
                pts[tuple(prefix)] = n
                n += 1
            return
        for i in range(sizes[len(prefix)]):
            rec(prefix + [i])
    rec([])
    return S.Lattice(tuple(sizes), pts)


def bowl(target):
    return lambda c: 1.0 + 0.1 * sum((a - b) ** 2 for a, b in zip(c, target))


def test_mutation_moves_one_coordinate_by_one_and_stays_on_built_points():
    lat = box([3, 2, 4], holes={(1, 1, 2)})
    rng = random.Random(1)
    x = (1, 1, 1)
    seen = set()
    for _ in range(500):
        y = S.mutate(lat, x, rng)
        assert y in lat.points
        diff = [abs(a - b) for a, b in zip(x, y)]
        assert sorted(diff) == [0, 0, 1]
        seen.add(y)
    assert (1, 1, 2) not in seen                       # the hole is never proposed
    assert seen == {(0, 1, 1), (2, 1, 1), (1, 0, 1), (1, 1, 0)}
    assert S.mutate(box([1, 1]), (0, 0), rng) is None  # no neighbour at all


def test_number_of_steps_follows_the_cooling_schedule():
    lat = box([5, 5])
    res = S.anneal(lat, (0, 0), bowl((4, 4)), lambda c: True, seed=3, t_max=0.05, t_min=5e-4, cool=1.05)
    assert len(res.steps) == math.ceil(math.log(0.05 / 5e-4) / math.log(1.05))
    temps = [s.temperature for s in res.steps]
    assert temps[0] == 0.05 and all(abs(b - a / 1.05) < 1e-15 for a, b in zip(temps, temps[1:]))
    assert temps[-1] > 5e-4


def test_deterministic_given_seed_and_different_across_seeds():
    lat = box([4, 4, 3])
    run = lambda seed: S.anneal(lat, (0, 0, 0), bowl((3, 2, 1)), lambda c: True, seed=seed)
    a, b, c = run(7), run(7), run(8)
    assert [s.candidate for s in a.steps] == [s.candidate for s in b.steps]
    assert a.best == b.best and a.t_best == b.t_best
    assert [s.candidate for s in a.steps] != [s.candidate for s in c.steps]


def test_finds_the_minimum_of_a_bowl_and_best_never_gets_worse():
    lat = box([6, 6])
    f = bowl((4, 1))
    res = S.anneal(lat, (0, 5), f, lambda c: True, seed=0, t_max=0.05, t_min=1e-5, cool=1.02)
    assert res.best == (4, 1) and res.t_best == 1.0
    e = [f(s.best) for s in res.steps]
    assert all(b <= a for a, b in zip(e, e[1:]))
    assert res.ranking()[0] == ((4, 1), 1.0)


def test_feedback_is_eq1_and_telescopes_over_accepted_moves():
    lat = box([5, 4])
    f = bowl((2, 3))
    res = S.anneal(lat, (0, 0), f, lambda c: True, seed=5)
    t0 = f((0, 0))
    total = 0.0
    for s in res.steps:
        assert s.feedback == pytest.approx((f(s.x) - f(s.candidate)) / t0)
        assert s.delta_e == pytest.approx(-s.feedback)
        if s.accepted:
            total += s.feedback
    assert total == pytest.approx((t0 - res.t_final) / t0)


def test_acceptance_rule_of_alg1():
    lat = box([2])
    # improvement: always accepted, best updated
    res = S.anneal(lat, (0,), lambda c: 2.0 if c == (0,) else 1.0, lambda c: True, seed=0)
    assert res.steps[0].accepted and res.steps[0].best == (1,)
    # Delta E = 0 goes to the else-branch and is always accepted (exp(0) = 1 > r); best unchanged
    res = S.anneal(lat, (0,), lambda c: 1.0, lambda c: True, seed=0)
    assert all(s.accepted and s.delta_e == 0 for s in res.steps)
    assert res.best == (0,)
    # a much worse candidate at a tiny temperature is never accepted
    res = S.anneal(lat, (0,), lambda c: 1.0 if c == (0,) else 2.0, lambda c: True, seed=0,
                   t_max=1e-3, t_min=1e-4, cool=1.5)
    assert not any(s.accepted for s in res.steps) and res.final == (0,)
    # at a huge temperature nearly everything is accepted
    res = S.anneal(lat, (0,), lambda c: 1.0 if c == (0,) else 1.01, lambda c: True, seed=0,
                   t_max=1e3, t_min=1e2, cool=1.01)
    up = [s for s in res.steps if s.delta_e and s.delta_e > 0]
    assert up and sum(s.accepted for s in up) >= 0.95 * len(up)


def test_variants_failing_admission_are_never_accepted_or_timed():
    lat = box([5])
    timed = []
    def measure(c):
        timed.append(c)
        return 10.0 - c[0]            # further right = faster
    res = S.anneal(lat, (0,), measure, lambda c: c[0] < 3, seed=2, t_max=0.5, t_min=1e-3, cool=1.03)
    assert all(c[0] < 3 for c in timed)
    assert res.best == (2,) and res.final[0] < 3
    assert (3,) in res.rejected and all(c[0] >= 3 for c in res.rejected)
    assert all(not s.accepted for s in res.steps if not s.admitted)
    with pytest.raises(ValueError):
        S.anneal(lat, (4,), measure, lambda c: c[0] < 3)        # x0 must pass its own test


def test_lattice_of_the_built_library_is_walkable():
    lat = S.Lattice.from_library(128, 1, True)
    assert len(lat.points) >= 2
    rng = random.Random(0)
    movable = [x for x in lat.points if S.mutate(lat, x, rng) is not None]
    assert movable, "no two built variants are lattice neighbours"
    f = lambda c: 1.0 + 0.01 * lat.points[c]
    res = S.anneal(lat, movable[0], f, lambda c: True, seed=1)
    assert res.best in lat.points and res.t_best <= res.t0


def test_store_resumes_a_killed_search_on_the_same_trajectory(tmp_path):
    """Sec. 4.1: every candidate is stored; a search that was cut short continues from the file
    to exactly the run it would have been, without repeating a measurement or a test."""
    lat = box([4, 4, 3], holes={(2, 2, 1)})
    x0 = (0, 0, 0)
    calls = {"measure": 0, "admit": 0}

    def measure(c):
        calls["measure"] += 1
        return bowl((3, 2, 1))(c) + 1e-3 * ((hash(c) % 7) - 3)

    def admit(c):
        calls["admit"] += 1
        return c != (1, 0, 0)

    header = {"workload": "toy", "seed": 5, "t_max": 0.05, "t_min": 5e-4, "cool": 1.05, "x0": list(x0)}
    full = S.anneal(lat, x0, measure, admit, seed=5)

    path = str(tmp_path / "search.jsonl")
    store = S.SearchStore(path, header)
    assert store.resume() == 0
    store.open(measure(x0))

    class Killed(Exception):
        pass

    def log_then_die(st):
        store.log(st)
        if st.step == 30:
            raise Killed

    with pytest.raises(Killed):
        S.anneal(lat, x0, measure, admit, seed=5, log=log_then_die)
    store.close()

    again = S.SearchStore(path, header)
    assert again.resume() == 31
    again.open(0.0)
    before = dict(calls)
    seen_before = set(again.known_times) | set(again.known_admitted)
    res = S.anneal(lat, x0, measure, admit, seed=5, log=again.log, known_times=again.known_times,
                   known_admitted=again.known_admitted)
    again.close()
    assert [(s.candidate, s.accepted, s.best) for s in res.steps] == [(s.candidate, s.accepted, s.best) for s in full.steps]
    assert res.best == full.best and res.t_best == full.t_best
    # nothing that was stored was measured or tested again
    new_points = {s.candidate for s in res.steps} - seen_before
    assert calls["measure"] - before["measure"] <= len(new_points)
    assert calls["admit"] - before["admit"] <= len(new_points)
    # the file now holds the whole run, each step once, and resumes to a finished search
    done = S.SearchStore(path, header)
    assert done.resume() == len(full.steps)
    # a store of another search is refused
    other = S.SearchStore(path, dict(header, seed=6))
    with pytest.raises(ValueError):
        other.resume()
