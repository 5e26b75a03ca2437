"""Pins of the scheduling oracle (adaptive batching, Alg. 1; token adaptation, Alg. 2 and Alg. 3) against
what the paper and the mathematics fix: hand-worked queues for each branch, the printed tables, exhaustive
enumeration on small queues, a replay of every returned plan, and planted mistakes that a pin must catch."""
import itertools
import math
import os
import random

import pytest

from oracle import otas_sched_oracle as so

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
GAMMAS = [-20, -15, -10, -5, 0, 2, 4, 8]          # Sec. V selection list
PAPER = dict(delta=0.5, epsilon=64, eta=0.5, mu=0.8)


def table1():
    rows = []
    for line in open(os.path.join(GOLD, "table1_rate_to_gamma.txt")):
        if line.startswith("#") or not line.strip():
            continue
        lo, hi, g = line.split()
        rows.append((float(lo), float(hi), int(g)))
    return rows


def table2():
    rows = []
    for line in open(os.path.join(GOLD, "table2_query_types.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, task, lat, u = line.split()
        rows.append((int(k), task, float(lat), float(u)))
    return rows


def Q(s, l, u, task=0):
    return so.Query(s=s, l=l, u=u, task=task)


# ------------------------------------------------------------------------------------------- Alg. 1
def test_alg1_first_query_opens_a_batch_and_compatible_query_joins_it():
    B = []
    assert so.add_query(B, Q(0.0, 1.0, 0.3), **PAPER) == 0
    assert so.add_query(B, Q(0.1, 1.0, 0.2), **PAPER) == 0
    assert len(B) == 1 and len(B[0].queries) == 2
    assert B[0].s == 0.0 and B[0].d == 1.0 and B[0].u == 0.3


def test_alg1_arrival_time_ends_the_walk():
    # The queue is in deadline order after a token-adaptation pass, so the last batch can be the one that
    # has waited longest.  It has waited more than delta: the walk ends there and a new batch is opened,
    # although the batch before it would accept r on every count.
    B = [so.Batch([Q(0.5, 0.6, 0.3)]), so.Batch([Q(0.0, 2.0, 0.3)])]
    assert so.add_query(B, Q(0.6, 0.6, 0.3), **PAPER) == 2
    # exactly at the limit (0.2 + 0.5 = 0.7, not < 0.7) the last batch still takes it
    B = [so.Batch([Q(0.0, 2.0, 0.3)]), so.Batch([Q(0.2, 2.0, 0.3)])]
    assert so.add_query(B, Q(0.7, 1.5, 0.3), **PAPER) == 1
    assert so.add_query(B, Q(0.71, 1.5, 0.3), **PAPER) == 2


def test_alg1_full_batch_is_skipped_for_an_older_one():
    full = so.Batch([Q(0.30, 1.0, 0.3) for _ in range(4)])
    B = [so.Batch([Q(0.25, 1.0, 0.3)]), full]
    assert so.add_query(B, Q(0.4, 0.9, 0.3), delta=0.5, epsilon=4, eta=0.5, mu=0.8) == 0
    assert len(B[0].queries) == 2 and len(B[1].queries) == 4


def test_alg1_deadline_and_utility_thresholds():
    B = [so.Batch([Q(0.0, 0.6, 0.3)])]
    # deadline 1.2 vs 0.6: 0.6 apart > eta
    assert so.add_query(B, Q(0.2, 1.0, 0.3), **PAPER) == 1
    # utility 1.2 vs u_b = 0.3: 0.9 apart > mu: skips batch 1 (d = 1.2) and batch 0, opens a third
    assert so.add_query(B, Q(0.2, 1.0, 1.2), **PAPER) == 2
    # close in deadline and utility to batch 0 only: newest-first walk skips 2 (utility) and 1 (deadline)
    assert so.add_query(B, Q(0.2, 0.45, 0.35), **PAPER) == 0
    # u_b stays the first query's utility, d_b follows the minimum deadline
    assert B[0].u == 0.3 and B[0].d == pytest.approx(0.6)
    # thresholds are strict: a difference equal to eta / mu is accepted
    B = [so.Batch([Q(0.0, 1.0, 0.25)])]
    assert so.add_query(B, Q(0.0, 1.5, 1.05), delta=0.5, epsilon=64, eta=0.5, mu=0.8) == 0


def test_alg1_invariants_on_a_random_trace():
    rng = random.Random(3)
    types = table2()
    B, t = [], 0.0
    for _ in range(3000):
        t += rng.expovariate(400.0)
        _, task, lat, u = rng.choice(types)
        so.add_query(B, Q(t, lat, u), **PAPER)
    assert sum(len(b.queries) for b in B) == 3000
    for b in B:
        first = b.queries[0]
        assert 1 <= len(b.queries) <= PAPER["epsilon"]
        assert [q.s for q in b.queries] == sorted(q.s for q in b.queries)
        for q in b.queries:
            assert q.s <= first.s + PAPER["delta"]
            assert abs(q.u - first.u) <= PAPER["mu"]
        # every joining query was within eta of the batch deadline at that moment, so all deadlines of a
        # batch lie within 2 eta of one another
        ds = [q.d for q in b.queries]
        assert max(ds) - min(ds) <= 2 * PAPER["eta"] + 1e-12


# ------------------------------------------------------------------------------------------- Table I / f
def test_rate_projection_reproduces_table1():
    rows = table1()
    f_table = [(hi, GAMMAS.index(g)) for _, hi, g in rows if math.isfinite(hi)]
    smallest = GAMMAS.index(min(GAMMAS))
    for lo, hi, g in rows:
        probes = [lo, lo + 1] + ([hi] if math.isfinite(hi) else [5000.0])
        for q in probes:
            assert GAMMAS[so.f_of_rate(q, f_table, smallest)] == g, (q, g)
    # the two rates the table leaves out take the row above them
    assert GAMMAS[so.f_of_rate(349, f_table, smallest)] == 0
    assert GAMMAS[so.f_of_rate(1000, f_table, smallest)] == -20


def test_rate_table_from_latency_gives_table1_back():
    """Table I read as the projection built from a latency profile: a model whose gamma serves `hi` requests per
    second (per-sample latency 1 / hi, two tasks of different speed with that mean) gets the table's rows back,
    the smallest gamma has no row, a gamma that is no faster than the one before it has none either, and the
    order of the selection list does not matter."""
    rows = table1()
    finite = [(hi, g) for _, hi, g in rows if math.isfinite(hi)]
    gammas = [g for _, g in finite] + [-20]                     # 8, 4, 2, 0, -5, -10, -15, -20
    mean_lat = [1.0 / hi for hi, _ in finite] + [1.0 / 5000.0]
    latency = [[0.5 * m for m in mean_lat], [1.5 * m for m in mean_lat]]      # mean over the tasks = 1 / hi
    got = so.rate_table_from_latency(gammas, latency)
    assert [gammas[i] for _, i in got] == [g for _, g in finite]
    assert [round(q, 6) for q, _ in got] == [hi for hi, _ in finite]
    for lo, hi, g in rows:
        for q in (lo, hi if math.isfinite(hi) else 5000.0):
            assert gammas[so.f_of_rate(q, got, gammas.index(-20))] == g
    # shuffled selection list: same rows (indices follow the list)
    perm = [3, 7, 0, 5, 1, 6, 2, 4]
    g2 = [gammas[i] for i in perm]
    lat2 = [[row[i] for i in perm] for row in latency]
    got2 = so.rate_table_from_latency(g2, lat2)
    assert [(round(q, 6), g2[i]) for q, i in got2] == [(round(q, 6), gammas[i]) for q, i in got]
    # gamma 2 made no faster than gamma 4: it loses its row
    slow = [list(r) for r in latency]
    for r in slow:
        r[2] = r[1]
    assert [gammas[i] for _, i in so.rate_table_from_latency(gammas, slow)] == [8, 4, 0, -5, -10, -15]


# ------------------------------------------------------------------------------------------- profile
def test_profile_counts_per_task_and_weights_utility():
    lat = [[0.001, 0.002], [0.010, 0.020]]
    acc = [[0.5, 0.9], [0.4, 0.8]]
    b = so.Batch([Q(0, 1, 1.0, 0), Q(0, 1, 0.2, 1), Q(0, 1, 0.3, 1)])
    t, U = so.profile(b, 1, lat, acc)
    assert t == pytest.approx(1 * 0.002 + 2 * 0.020)
    assert U == pytest.approx(1.0 * 0.9 + 0.2 * 0.8 + 0.3 * 0.8)


# ------------------------------------------------------------------------------------------- Alg. 3
def test_alg3_hand_worked_queue():
    gam = [-10, 0, 8]
    lat = [[0.001, 0.002, 0.004]]                      # one task, per-sample seconds at each gamma
    acc = [[0.7, 0.9, 0.95]]
    f_table = [(100.0, 2), (300.0, 1)]                 # q <= 100 -> gamma 8, q <= 300 -> gamma 0, else min
    mk = lambda n, s, l, u: so.Batch([Q(s, l, u) for _ in range(n)])
    # q = 200 -> gamma 0 (2 ms / sample).  T = 0.
    B = [mk(50, 0.0, 0.15, 0.3),      # 0 + 0.100 < 0.15, mean u 0.3 <= kappa -> gamma 0, T = 0.100
         mk(50, 0.0, 0.18, 0.3),      # 0.100 + 0.100 >= 0.18 -> min gamma, T = 0.150
         mk(10, 0.0, 1.00, 0.9),      # 0.150 + 0.020 < 1.0, mean u 0.9 > kappa -> max gamma, T = 0.190
         mk(10, 0.0, 0.21, 0.9)]      # 0.190 + 0.020 >= 0.21 -> min gamma (deadline rule comes first)
    so.manually_allocate(B, 0.0, gam, 200.0, f_table, 0.8, lat, acc)
    assert [gam[b.gamma] for b in B] == [0, -10, 8, -10]
    # a rate beyond the table falls to the smallest gamma for every batch that is not high-utility
    B = [mk(5, 0.0, 1.0, 0.3), mk(5, 0.0, 1.0, 0.9)]
    so.manually_allocate(B, 0.0, gam, 1e9, f_table, 0.8, lat, acc)
    assert [gam[b.gamma] for b in B] == [-10, 8]


# ------------------------------------------------------------------------------------------- Alg. 2
def random_queue(rng, nb, n_tasks, tight):
    B = []
    for _ in range(nb):
        n = rng.randint(1, 6)
        s = rng.uniform(0.0, 0.2)
        l = rng.uniform(0.05, 0.25) if tight else 1e6
        B.append(so.Batch([Q(s, l, rng.choice([0.01, 0.2, 0.3, 1.0]), rng.randrange(n_tasks)) for _ in range(n)]))
    return B


def random_tables(rng, n_tasks, ng):
    lat = [sorted(rng.uniform(0.002, 0.02) for _ in range(ng)) for _ in range(n_tasks)]
    acc = [sorted(rng.uniform(0.3, 0.99) for _ in range(ng)) for _ in range(n_tasks)]
    return lat, acc


def brute_force(B, T, ng, lat, acc):
    """The optimum of the batch-level problem (Eq. 3 with every request of a batch sharing its fate):
    every assignment of {not executed, gamma_1..gamma_N} to the deadline-sorted queue, executed in order."""
    best = -math.inf
    for choice in itertools.product(range(ng + 1), repeat=len(B)):
        clock, total, ok = T, 0.0, True
        for b, c in zip(B, choice):
            if c == 0:
                continue
            t, U = so.profile(b, c - 1, lat, acc)
            if clock + t < b.d:
                clock += t
                total += U
            else:
                ok = False
                break
        if ok:
            best = max(best, total)
    return best


def test_alg2_takes_alg3_for_short_queues_and_in_the_initial_stage():
    rng = random.Random(5)
    lat, acc = random_tables(rng, 2, 3)
    f_table = [(100.0, 2), (300.0, 1)]
    for nb, initial in [(3, False), (5, False), (8, True)]:
        B = random_queue(rng, nb, 2, tight=True)
        ref = sorted([so.Batch(list(b.queries)) for b in B], key=lambda b: b.d)
        so.manually_allocate(ref, 0.05, [-10, 0, 8], 200.0, f_table, 0.8, lat, acc)
        out = so.allocate(B, 0.05, [-10, 0, 8], 200.0, 5, initial, f_table, 0.8, lat, acc)
        assert math.isnan(out)
        assert [b.gamma for b in B] == [b.gamma for b in ref]
        assert [b.d for b in B] == sorted(b.d for b in B)


def test_alg2_is_optimal_when_deadlines_do_not_bind():
    rng = random.Random(7)
    for trial in range(20):
        ng = rng.randint(2, 4)
        lat, acc = random_tables(rng, 3, ng)
        # accuracy not monotone in gamma for some tasks, so "largest gamma" is not always the answer
        for row in acc:
            rng.shuffle(row)
        B = random_queue(rng, 6, 3, tight=False)
        best = so.allocate(B, 0.0, list(range(ng)), 0.0, 5, False, [], 0.8, lat, acc)
        want = 0.0
        for b in B:
            want += max(so.profile(b, g, lat, acc)[1] for g in range(ng))
        assert best == pytest.approx(want, rel=1e-12)
        for b in B:
            assert b.gamma is not None
            assert so.profile(b, b.gamma, lat, acc)[1] == max(so.profile(b, g, lat, acc)[1] for g in range(ng))


def test_alg2_plans_are_feasible_replay_to_their_value_and_never_beat_the_optimum():
    rng = random.Random(11)
    hits = 0
    for trial in range(60):
        ng = rng.randint(2, 3)
        lat, acc = random_tables(rng, 2, ng)
        B = random_queue(rng, 6, 2, tight=True)
        T = rng.uniform(0.0, 0.05)
        best = so.allocate(B, T, list(range(ng)), 0.0, 5, False, [], 0.8, lat, acc)
        got, _, ok = so.replay(B, T, lat, acc)
        assert ok                                        # every executed batch meets its deadline
        assert got == pytest.approx(best, rel=1e-12, abs=1e-15)
        opt = brute_force(B, T, ng, lat, acc)
        assert best <= opt + 1e-12
        hits += abs(best - opt) <= 1e-12
        dropped = [b for b in B if b.gamma is None]
        assert len(dropped) < len(B) or opt == 0.0
    assert hits >= 30          # the table keeps one plan per (b, l_b): a heuristic, but right most of the time


def test_alg2_single_gamma_reduces_to_deadline_scheduling_with_rejection():
    # one gamma, equal utilities per request and unit accuracy: the plan's value is the number of requests
    # served, and the dynamic program may only drop batches.  With a queue whose first batch is too slow to
    # let the second finish, but whose second alone is worth more, the plan drops the first.
    lat, acc = [[0.01]], [[1.0]]
    mk = lambda n, d: so.Batch([Q(0.0, d, 1.0) for _ in range(n)])
    B = [mk(10, 0.11), mk(30, 0.35), mk(1, 10.0), mk(1, 10.0), mk(1, 10.0), mk(1, 10.0)]
    best = so.allocate(B, 0.0, [0], 0.0, 5, False, [], 0.8, lat, acc)
    # executing batch 0 (0.10 s) leaves batch 1 (0.30 s) finishing at 0.40 >= 0.35
    assert [b.gamma for b in B] == [None, 0, 0, 0, 0, 0]
    assert best == pytest.approx(34.0)


def test_alg2_hopeless_head_batches_are_skipped_not_executed():
    # the first two batches cannot finish under any gamma: every state that skips them has accumulated
    # utility exactly 0, the case in which the listing's initial S = 1 would name an infeasible predecessor
    lat, acc = [[0.01, 0.02]], [[0.8, 0.9]]
    mk = lambda n, d, u=1.0: so.Batch([Q(0.0, d, u) for _ in range(n)])
    B = [mk(10, 0.05), mk(10, 0.06), mk(5, 1.0), mk(5, 1.1), mk(5, 1.2), mk(5, 1.3)]
    T = 0.0
    best = so.allocate(B, T, [0, 8], 0.0, 5, False, [], 0.8, lat, acc)
    assert [b.gamma for b in B] == [None, None, 1, 1, 1, 1]
    got, clock, ok = so.replay(B, T, lat, acc)
    assert ok and got == pytest.approx(best) and best == pytest.approx(20 * 0.9)
    assert clock == pytest.approx(20 * 0.02)
    # zero-utility requests: the plan still carries the clock through the batches it executes
    B = [mk(10, 0.25, 0.0), mk(10, 0.25, 0.0), mk(5, 0.30), mk(1, 9.0), mk(1, 9.0), mk(1, 9.0)]
    best = so.allocate(B, 0.0, [0, 8], 0.0, 5, False, [], 0.8, lat, acc)
    got, clock, ok = so.replay(B, 0.0, lat, acc)
    assert ok and got == pytest.approx(best)


# ------------------------------------------------------------------------------------------- planted mistakes
def test_planted_mistakes_are_caught():
    """Each plausible slip, planted in the oracle, fails at least one of the pins above."""
    import types

    def fails(test, *a):
        try:
            test(*a)
        except AssertionError:
            return True
        return False

    real = globals()["so"]
    src = open(real.__file__).read()

    def variant(old, new):
        assert old in src
        mod = types.ModuleType("planted")
        mod.__dict__["__name__"] = "planted"
        exec(compile(src.replace(old, new).replace("from __future__ import annotations\n", ""), "planted", "exec"),
             mod.__dict__)
        return mod

    plants = [
        ("for b in range(len(B) - 1, -1, -1):", "for b in range(len(B)):",                      # oldest-first walk
         [test_alg1_deadline_and_utility_thresholds, test_alg1_arrival_time_ends_the_walk]),
        ("if B[b].s + delta < r.s:               # arrival time: the batch has waited too long\n            break",
         "if B[b].s + delta < r.s:\n            continue",                                       # break -> continue
         [test_alg1_arrival_time_ends_the_walk]),
        ("elif abs(B[b].d - r.d) > eta:", "elif abs(B[b].s - r.d) > eta:",                       # wrong field
         [test_alg1_deadline_and_utility_thresholds]),
        ("if C[b - 1][lp] + t < B[b - 1].d:", "if T + t < B[b - 1].d:",                          # clock not carried
         [test_alg2_plans_are_feasible_replay_to_their_value_and_never_beat_the_optimum,
          test_alg2_single_gamma_reduces_to_deadline_scheduling_with_rejection]),
        ("l = S[b + 1][l]", "l = S[b][l]",                                                       # backtrack off by one
         [test_alg2_plans_are_feasible_replay_to_their_value_and_never_beat_the_optimum,
          test_alg2_single_gamma_reduces_to_deadline_scheduling_with_rejection]),
        ("if T + t >= b.d:\n            b.gamma = g_min", "if T + t >= b.d:\n            b.gamma = g_max",
         [test_alg3_hand_worked_queue]),
        ("        T = T + t\n", "        T = T\n", [test_alg3_hand_worked_queue]),               # Alg. 3 clock frozen
        ("U += q.u * accuracy[q.task][g]", "U += accuracy[q.task][g]",                           # utility weight lost
         [test_profile_counts_per_task_and_weights_utility]),
    ]
    try:
        for old, new, tests in plants:
            globals()["so"] = variant(old, new)
            assert any(fails(t) for t in tests), old
    finally:
        globals()["so"] = real
