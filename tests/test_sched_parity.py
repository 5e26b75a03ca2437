"""The library's host scheduler (C ABI of include/otas_sched.h) against the scheduling oracle: every decision
(which batch takes a request, the queue order after a pass, the gamma of every batch) and every reported double
(batch aggregates, estimates, planned utility) must be identical, on seeded traces shaped like the paper's
synthetic workload.  Host code only: runs without a GPU."""
import math
import random

import numpy as np
import pytest

import otas_synth as synth
import paper_2401_05031_amd as otas
from oracle import otas_sched_oracle as so
from paper_2401_05031_amd import serve

GAMMAS = list(synth.GAMMA_LIST)


def _ensure_built():
    import os
    if not os.path.exists(otas.lib_path()):
        from paper_2401_05031_amd import build
        build.build(verbose=False)


def tables(seed, n_tasks=3, scale=1.0):
    rng = np.random.default_rng(seed)
    # per-sample latency falls as more tokens are merged and rises with prompts, as the paper profiles
    base = rng.uniform(0.0015, 0.0025, size=(n_tasks, 1)) * scale
    lat = base * np.array([0.55, 0.65, 0.77, 0.88, 1.0, 1.01, 1.02, 1.05])[None, :]
    acc = synth.stand_in_accuracy(GAMMAS, n_tasks)
    return lat, acc


class OracleScheduler:
    """The oracle behind the method names the serving loop uses."""

    def __init__(self, gammas, lat, acc, rate_table, delta=0.5, epsilon=64, eta=0.5, mu=0.8, beta=5, kappa=0.8):
        self.gammas, self.lat, self.acc, self.rate = list(gammas), [list(r) for r in lat], [list(r) for r in acc], rate_table
        self.p = dict(delta=delta, epsilon=epsilon, eta=eta, mu=mu)
        self.beta, self.kappa = beta, kappa
        self.B = []

    def otas_sched_add_query(self, id, s_r, l_r, u_r, task):
        q = so.Query(s_r, l_r, u_r, task)
        q.id = id
        return so.add_query(self.B, q, **self.p)

    def otas_sched_allocate(self, T, q, initial):
        if not self.B:
            return float("nan")
        return so.allocate(self.B, T, self.gammas, q, self.beta, initial, self.rate, self.kappa, self.lat, self.acc)

    def otas_sched_num_batches(self):
        return len(self.B)

    def otas_sched_batch_info(self, b):
        bt = self.B[b]
        g = bt.gamma
        if g is None:
            g = otas.OTAS_GAMMA_SKIP if getattr(bt, "seen", False) else otas.OTAS_GAMMA_UNDECIDED
        return {"size": len(bt.queries), "s_b": bt.s, "d_b": bt.d, "u_b": bt.u, "gamma_index": g}

    def otas_sched_batch_queries(self, b):
        return [q.id for q in self.B[b].queries], [q.task for q in self.B[b].queries]

    def otas_sched_estimate(self, b, g):
        return so.profile(self.B[b], g, self.lat, self.acc)

    def otas_sched_remove(self, b):
        del self.B[b]


def same_queue(lib, orc, check_gamma=True):
    assert lib.otas_sched_num_batches() == orc.otas_sched_num_batches()
    for b in range(lib.otas_sched_num_batches()):
        a, o = lib.otas_sched_batch_info(b), orc.otas_sched_batch_info(b)
        if not check_gamma:
            a.pop("gamma_index"), o.pop("gamma_index")
        elif o["gamma_index"] == otas.OTAS_GAMMA_UNDECIDED and orc.B[b].gamma is None:
            o["gamma_index"] = a["gamma_index"]       # the oracle has one "None" for skipped and undecided
        assert a == o, (b, a, o)                       # doubles compared exactly
        assert lib.otas_sched_batch_queries(b) == orc.otas_sched_batch_queries(b)


@pytest.mark.parametrize("seed,rate", [(1, (200, 700)), (2, (900, 1500)), (3, (20, 60))])
def test_batching_and_allocation_match_the_oracle(seed, rate):
    _ensure_built()
    lat, acc = tables(seed)
    rate_table = serve.rate_table_from_latency(GAMMAS, lat)
    lib = otas.Scheduler(GAMMAS, lat, acc, rate_table)
    orc = OracleScheduler(GAMMAS, lat, acc, rate_table)
    trace = synth.poisson_trace(seed, 6, *rate)
    rng = random.Random(seed)
    next_pass = 0.3
    passes = dp_passes = skipped = 0
    for i, (s, l, u, task) in enumerate(trace):
        assert lib.otas_sched_add_query(i, s, l, u, task) == orc.otas_sched_add_query(i, s, l, u, task)
        if s >= next_pass:
            next_pass = s + rng.uniform(0.05, 0.4)
            T = s + rng.uniform(0.0, 0.3)           # a clock ahead of the arrivals makes deadlines bind
            q = rng.uniform(100, 1500)
            initial = rng.random() < 0.15
            a, o = lib.otas_sched_allocate(T, q, initial), orc.otas_sched_allocate(T, q, initial)
            assert (math.isnan(a) and math.isnan(o)) or a == o
            same_queue(lib, orc)
            passes += 1
            dp_passes += not math.isnan(a)
            for b in range(lib.otas_sched_num_batches()):
                for g in (0, len(GAMMAS) - 1):
                    assert lib.otas_sched_estimate(b, g) == orc.otas_sched_estimate(b, g)
                skipped += lib.otas_sched_batch_info(b)["gamma_index"] == otas.OTAS_GAMMA_SKIP
            # the engine takes some batches away
            for _ in range(rng.randint(0, 3)):
                if lib.otas_sched_num_batches():
                    b = rng.randrange(lib.otas_sched_num_batches())
                    lib.otas_sched_remove(b), orc.otas_sched_remove(b)
    same_queue(lib, orc, check_gamma=False)
    assert passes >= 10
    if rate[0] >= 200:
        assert dp_passes >= 5 and skipped > 0      # the dynamic program ran and had to drop batches


def test_paper_settings_batches_respect_thresholds():
    _ensure_built()
    lat, acc = tables(4)
    lib = otas.Scheduler(GAMMAS, lat, acc)
    trace = synth.poisson_trace(9, 4)
    for i, (s, l, u, task) in enumerate(trace):
        lib.otas_sched_add_query(i, s, l, u, task)
    total = 0
    for b in range(lib.otas_sched_num_batches()):
        info = lib.otas_sched_batch_info(b)
        ids, tasks = lib.otas_sched_batch_queries(b)
        total += len(ids)
        assert 1 <= info["size"] == len(ids) <= 64
        assert info["gamma_index"] == otas.OTAS_GAMMA_UNDECIDED
        assert info["s_b"] == trace[ids[0]][0] and info["u_b"] == trace[ids[0]][2]
        assert info["d_b"] == min(trace[i][0] + trace[i][1] for i in ids)
        assert all(trace[i][0] <= info["s_b"] + 0.5 for i in ids)
        assert [trace[i][3] for i in ids] == tasks
    assert total == len(trace)


def test_argument_errors():
    _ensure_built()
    lat, acc = tables(5)
    with pytest.raises(otas.OtasError):
        otas.Scheduler([0, 0], lat[:, :2], acc[:, :2])                       # repeated gamma
    with pytest.raises(otas.OtasError):
        otas.Scheduler(GAMMAS, -lat, acc)                                    # non-positive latency
    with pytest.raises(otas.OtasError):
        otas.Scheduler(GAMMAS, lat, acc, [(300.0, 1), (200.0, 2)])           # rates not ascending
    with pytest.raises(otas.OtasError):
        otas.Scheduler(GAMMAS, lat, acc, [(300.0, 8)])                       # gamma index out of range
    with pytest.raises(otas.OtasError):
        otas.Scheduler(GAMMAS, lat, acc, epsilon=0)
    s = otas.Scheduler(GAMMAS, lat, acc)
    with pytest.raises(otas.OtasError):
        s.otas_sched_add_query(0, 0.0, 1.0, 0.3, 3)                          # unknown task
    with pytest.raises(otas.OtasError):
        s.otas_sched_add_query(0, float("nan"), 1.0, 0.3, 0)
    assert math.isnan(s.otas_sched_allocate(0.0, 100.0, False)) and s.otas_sched_num_batches() == 0
    with pytest.raises(otas.OtasError):
        s.otas_sched_batch_info(0)
    with pytest.raises(otas.OtasError):
        s.otas_sched_remove(0)
    s.otas_sched_add_query(7, 0.0, 1.0, 0.3, 1)
    with pytest.raises(otas.OtasError):
        s.otas_sched_estimate(0, len(GAMMAS))
    assert s.otas_sched_batch_queries(0) == ([7], [1])


def test_rate_table_library_equals_oracle_exactly():
    """otas_sched_rate_table against the oracle's statement of the projection: identical rows (exact
    doubles), also with unsorted gamma lists, a gamma no faster than its neighbour (no row) and one task."""
    _ensure_built()
    from oracle import otas_sched_oracle as so
    rng = np.random.default_rng(3)
    for n_tasks in (1, 3, 6):
        for gl in (GAMMAS, [0], [-5, 8, 0, -20, 4], list(reversed(GAMMAS))):
            lat = rng.uniform(1e-4, 2e-3, size=(n_tasks, len(gl)))
            if len(gl) > 2:
                lat[:, 1] = lat[:, 0]                 # equal throughput: the later one gets no row
            want = so.rate_table_from_latency(gl, lat.tolist())
            got = otas.otas_sched_rate_table(gl, lat)
            assert got == want
    # the paper's Table I is such a projection: throughputs 279, 319, ... give its rows back
    gl = [8, 4, 2, 0, -5, -10, -15, -20]
    thr = [279.0, 319.0, 348.0, 379.0, 449.0, 519.0, 999.0, 5000.0]
    lat = np.array([[1.0 / t for t in thr]])
    rows = otas.otas_sched_rate_table(gl, lat)
    assert [g for _, g in rows] == list(range(7)) and [round(r) for r, _ in rows] == [279, 319, 348, 379, 449, 519, 999]
    with pytest.raises(otas.OtasError):
        otas.otas_sched_rate_table(gl, np.zeros((1, 8)))


def test_rate_table_from_latency_orders_gammas_by_throughput():
    lat, _ = tables(6)
    rows = serve.rate_table_from_latency(GAMMAS, lat)
    assert [GAMMAS[g] for _, g in rows] == [8, 4, 2, 0, -5, -10, -15]        # the smallest gamma is the overflow
    assert all(rows[i][0] < rows[i + 1][0] for i in range(len(rows) - 1))
    thr8 = 1.0 / np.mean(lat[:, GAMMAS.index(8)])
    assert rows[0][0] == pytest.approx(thr8)


@pytest.mark.parametrize("load", [0.5, 1.0, 1.6])
def test_serving_loop_same_decisions_with_either_scheduler(load):
    """The loop driven by the library's scheduler and by the oracle: identical run / give-up records; and the
    loop's accounting adds up."""
    _ensure_built()
    lat, acc = tables(8)
    rate_table = serve.rate_table_from_latency(GAMMAS, lat)
    thr0 = 1.0 / np.mean(lat[:, GAMMAS.index(0)])           # requests / s of the plain model
    trace = synth.poisson_trace(12, 8, 0.45 * load * thr0, 1.55 * load * thr0)
    eng = serve.ProfileEngine(lat)
    a = serve.replay_trace(otas.Scheduler(GAMMAS, lat, acc, rate_table), trace, eng, acc, log=True)
    o = serve.replay_trace(OracleScheduler(GAMMAS, lat, acc, rate_table), trace, eng, acc, log=True)
    assert a["log"] == o["log"] and a["utility"] == o["utility"]
    assert a["served"] + a["late"] + a["given_up"] == len(trace)
    assert 0.0 < a["utility"] <= a["offered_utility"]
    ran = [rec for rec in a["log"] if rec[0] == "run"]
    assert all(ran[k][1] + ran[k][4] <= ran[k + 1][1] + 1e-12 for k in range(len(ran) - 1))   # one batch at a time
    seen = sorted(i for rec in a["log"] for i in rec[2])
    assert seen == list(range(len(trace)))
    if load <= 0.5:
        assert a["given_up"] == 0 and a["late"] == 0
        assert a["gamma_batches"][8] == max(a["gamma_batches"].values())        # light load: prompts everywhere
    if load >= 1.6:
        assert sum(v for g, v in a["gamma_batches"].items() if g < 0) > 0 and a["given_up"] > 0   # overload: merge, drop


def test_token_adaptation_beats_a_fixed_gamma_under_fluctuating_load():
    """What the paper's evaluation shows qualitatively (Sec. V, main results): adapting gamma earns more utility
    than serving every batch with the plain model, under a load that swings around the plain model's capacity."""
    _ensure_built()
    lat, acc = tables(10)
    thr0 = 1.0 / np.mean(lat[:, GAMMAS.index(0)])
    trace = synth.poisson_trace(21, 12, 0.5 * thr0, 1.7 * thr0)
    eng = serve.ProfileEngine(lat)
    adaptive = serve.replay_trace(otas.Scheduler(GAMMAS, lat, acc, serve.rate_table_from_latency(GAMMAS, lat)), trace, eng, acc)
    i0 = GAMMAS.index(0)
    fixed = serve.replay_trace(otas.Scheduler([0], lat[:, i0:i0 + 1], acc[:, i0:i0 + 1]), trace,
                               serve.ProfileEngine(lat[:, i0:i0 + 1]), acc[:, i0:i0 + 1])
    assert adaptive["utility"] > fixed["utility"]


@pytest.mark.parametrize("params", [dict(delta=0.1, epsilon=4, eta=0.05, mu=0.1, beta=2, kappa=0.25),
                                    dict(delta=2.0, epsilon=200, eta=5.0, mu=5.0, beta=0, kappa=0.0)])
def test_other_thresholds_match_the_oracle(params):
    """Thresholds far from the paper's: tiny batches split on every criterion, and one where nearly everything
    joins one batch and the dynamic program runs on every pass (beta = 0)."""
    _ensure_built()
    lat, acc = tables(31)
    rate_table = serve.rate_table_from_latency(GAMMAS, lat)
    lib = otas.Scheduler(GAMMAS, lat, acc, rate_table, **params)
    orc = OracleScheduler(GAMMAS, lat, acc, rate_table, **params)
    trace = synth.poisson_trace(33, 3, 150, 400)
    rng = random.Random(7)
    for i, (s, l, u, task) in enumerate(trace):
        assert lib.otas_sched_add_query(i, s, l, u, task) == orc.otas_sched_add_query(i, s, l, u, task)
        if i % 97 == 96:
            T = s + rng.uniform(0.0, 0.2)
            a, o = lib.otas_sched_allocate(T, 300.0, False), orc.otas_sched_allocate(T, 300.0, False)
            assert (math.isnan(a) and math.isnan(o)) or a == o
            same_queue(lib, orc)
            for _ in range(min(3, lib.otas_sched_num_batches())):
                lib.otas_sched_remove(0), orc.otas_sched_remove(0)
    same_queue(lib, orc, check_gamma=False)
    sizes = [lib.otas_sched_batch_info(b)["size"] for b in range(lib.otas_sched_num_batches())]
    assert max(sizes) <= params["epsilon"]


def test_allocator_scales_to_long_queues():
    """2000 queued batches, 8 gammas: one pass of the dynamic program stays in the milliseconds (it is linear in the
    queue length) and returns a feasible plan."""
    import time
    _ensure_built()
    lat, acc = tables(41)
    lib = otas.Scheduler(GAMMAS, lat, acc, delta=0.0, epsilon=1)        # every request its own batch
    rng = np.random.default_rng(5)
    t = 0.0
    for i in range(2000):
        t += rng.exponential(1 / 2000.0)
        lib.otas_sched_add_query(i, t, float(rng.uniform(0.5, 3.0)), float(rng.choice([0.01, 0.2, 0.3, 1.0])), int(rng.integers(3)))
    assert lib.otas_sched_num_batches() == 2000
    t0 = time.perf_counter()
    best = lib.otas_sched_allocate(t, 2000.0, False)
    dt = time.perf_counter() - t0
    assert dt < 0.25 and best > 0
    clock, total = t, 0.0
    for b in range(2000):
        info = lib.otas_sched_batch_info(b)
        if b:
            assert info["d_b"] >= lib.otas_sched_batch_info(b - 1)["d_b"]
        if info["gamma_index"] >= 0:
            th, U = lib.otas_sched_estimate(b, info["gamma_index"])
            clock += th
            assert clock < info["d_b"]
            total += U
    assert total == pytest.approx(best, rel=1e-9)
