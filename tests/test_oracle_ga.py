"""Pins for the genetic-search oracle (CPU only): what eqs. (1)-(2) and the step
descriptions of Section 2.3 "Genetic search" fix, plus published splitmix64 outputs and
exhaustive search on small spaces."""
import itertools
import math

import pytest

from oracle import ga


def test_splitmix64_published_vectors():
    # first outputs for seed 0 as listed with the reference description of splitmix64
    r = ga.SplitMix64(0)
    assert [r.next_u64() for _ in range(3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4,
                                                0x06C45D188009454F]
    r = ga.SplitMix64(1234567)
    assert [r.next_u64() for _ in range(2)] == [6457827717110365317, 3203168211198807973]


def test_uniform_and_randint_ranges():
    r = ga.SplitMix64(7)
    us = [r.uniform() for _ in range(20000)]
    assert 0.0 <= min(us) and max(us) < 1.0
    assert abs(sum(us) / len(us) - 0.5) < 0.01
    vals = [r.randint(-2, 3) for _ in range(6000)]
    assert set(vals) == {-2, -1, 0, 1, 2, 3}
    for v in range(-2, 4):
        assert abs(vals.count(v) - 1000) < 150


def test_eq1_probabilities():
    f = [3.0, 1.0, 0.0, 4.0]
    p = ga.selection_probabilities(f)
    assert p == [0.375, 0.125, 0.0, 0.5]
    assert abs(sum(ga.selection_probabilities([0.1 * i for i in range(1, 40)])) - 1.0) < 1e-12
    assert ga.selection_probabilities([0.0, 0.0]) == [0.5, 0.5]


def test_eq2_cumulative_is_monotone_and_ends_at_one():
    p = ga.selection_probabilities([0.3, 0.1, 0.7, 0.05, 0.2])
    P = ga.cumulative_probabilities(p)
    assert all(b >= a for a, b in zip(P, P[1:]))
    assert P[-1] == 1.0
    for i in range(len(p)):
        assert abs(P[i] - sum(p[:i + 1])) < 1e-15


def test_roulette_interval_rule():
    P = [0.25, 0.25, 0.75, 1.0]          # second individual has probability 0
    assert ga.roulette_pick(P, 0.0) == 0          # v = 0 picks the first
    assert ga.roulette_pick(P, 0.25) == 0         # P(a_0) < v <= P(a_1)
    assert ga.roulette_pick(P, 0.2500001) == 2    # zero-width interval is never picked
    assert ga.roulette_pick(P, 0.75) == 2
    assert ga.roulette_pick(P, 0.7500001) == 3
    assert ga.roulette_pick(P, 1.0) == 3


def test_roulette_frequencies_follow_p():
    f = [5.0, 3.0, 1.0, 1.0]
    P = ga.cumulative_probabilities(ga.selection_probabilities(f))
    r = ga.SplitMix64(99)
    n = 40000
    counts = [0] * 4
    for _ in range(n):
        counts[ga.roulette_pick(P, r.uniform())] += 1
    chi2 = sum((c - n * fi / 10.0) ** 2 / (n * fi / 10.0) for c, fi in zip(counts, f))
    assert chi2 < 16.27      # chi-square, 3 dof, p = 0.001


def test_sort_is_descending_and_stable():
    assert ga.sort_by_fitness([1.0, 3.0, 3.0, 0.5, 2.0]) == [1, 2, 4, 0, 3]


LO, HI = [0, 0, 0, 0], [7, 5, 9, 3]
TARGET = (5, 2, 7, 1)


def separable(ch):
    # "runtime" grows with the distance from TARGET; fitness = 1 / runtime
    return 1.0 / (1.0 + sum((a - b) ** 2 for a, b in zip(ch, TARGET)))


def even_sum(ch):
    return sum(ch) % 2 == 0


def test_elites_survive_and_best_is_monotone():
    res = ga.genetic_search(LO, HI, even_sum, separable, seed=3, pop=16, elites=3, eps=0.0,
                            patience=100, max_gen=12)
    hist = res["history"]
    assert len(hist) == 12
    best = -1.0
    for (pop, fit), (npop, _) in zip(hist, hist[1:]):
        order = ga.sort_by_fitness(fit)
        assert npop[:3] == [pop[i] for i in order[:3]]
        assert max(fit) >= best
        best = max(fit)
    for pop, fit in hist:
        assert all(even_sum(ch) for ch in pop)
        assert all(all(l <= g <= h for g, l, h in zip(ch, LO, HI)) for ch in pop)
        assert fit == [separable(ch) for ch in pop]
    assert res["best_fitness"] == max(max(f) for _, f in hist)


def test_finds_the_optimum_of_a_separable_fitness():
    hits = 0
    for seed in range(10):
        res = ga.genetic_search(LO, HI, lambda ch: True, separable, seed=seed, pop=32,
                                elites=4, eps=0.0, patience=8, max_gen=30)
        hits += res["best"] == TARGET
    assert hits >= 8


def test_close_to_exhaustive_and_not_worse_than_random_at_equal_budget():
    # rugged, non-separable fitness on a 8*6*10*4 = 1920-point space
    def rugged(ch):
        a, b, c, d = ch
        t = 1.0 + abs(a * b - 12) + 0.5 * abs(c - 2 * d) + ((a + c) % 3) * 0.7
        return 1.0 / t
    space = list(itertools.product(*[range(l, h + 1) for l, h in zip(LO, HI)]))
    best_exh = max(rugged(ch) for ch in space)
    ga_scores, rnd_scores = [], []
    for seed in range(12):
        res = ga.genetic_search(LO, HI, lambda ch: True, rugged, seed=seed, pop=24, elites=3,
                                eps=0.0, patience=6, max_gen=20)
        ga_scores.append(res["best_fitness"])
        rng = ga.SplitMix64(1000 + seed)
        seen = set()
        while len(seen) < res["evaluations"]:
            seen.add(ga.random_legal(rng, LO, HI, lambda ch: True))
        rnd_scores.append(max(rugged(ch) for ch in seen))
    # the optimum is a needle (fitness 1.0, next best 0.67): a heuristic search finds it in
    # most runs, not all, and on average does at least as well as random draws
    assert sum(s >= 0.97 * best_exh for s in ga_scores) >= 7
    assert sum(ga_scores) / 12 >= sum(rnd_scores) / 12
    assert min(ga_scores) >= 0.5 * best_exh


def test_convergence_rule_on_runtimes():
    assert ga.runtimes_close([1.0, 1.0 / 1.04, 1.0 / 1.01], 0.05)
    assert not ga.runtimes_close([1.0, 1.0 / 1.06], 0.05)
    assert not ga.runtimes_close([1.0, 0.0], 0.05)
    # a flat fitness converges in the first generation
    res = ga.genetic_search(LO, HI, lambda ch: True, lambda ch: 2.0, seed=0, pop=8, elites=2)
    assert len(res["history"]) == 1


def test_varying_population_size_and_participants():
    res = ga.genetic_search(LO, HI, lambda ch: True, separable, seed=5, pop=20, elites=2,
                            next_pop=12, participants=6, eps=0.0, patience=50, max_gen=4)
    sizes = [len(p) for p, _ in res["history"]]
    assert sizes == [20, 12, 12, 12]


def test_same_seed_same_run():
    a = ga.genetic_search(LO, HI, even_sum, separable, seed=11, pop=12, elites=2, max_gen=6)
    b = ga.genetic_search(LO, HI, even_sum, separable, seed=11, pop=12, elites=2, max_gen=6)
    c = ga.genetic_search(LO, HI, even_sum, separable, seed=12, pop=12, elites=2, max_gen=6)
    assert a["history"] == b["history"]
    assert a["history"] != c["history"]
