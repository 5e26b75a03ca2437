"""CPU oracle for the host side of OTAS: adaptive batching (Sec. III-C, Alg. 1) and online token
adaptation (Sec. III-D, Alg. 2 with its fallback Alg. 3 and the profile-based estimates).

TEST INFRASTRUCTURE ONLY: plain Python, the algorithms' steps in the paper's order and notation.
The library's scheduler (csrc/sched.cpp) shares no code with it.

Notation (Sec. III-C): a request r has arrival time s_r, latency requirement l_r, finish deadline
d_r = s_r + l_r and utility u_r, and belongs to a task.  A batch b has s_b = min s_r, d_b = min d_r,
and u_b = the utility of its first arrived request.  gamma values come from a selection list
L^(gamma); a batch may also stay unexecuted.

Readings taken where the paper is silent or garbled:
  S1  Alg. 1 walks the batch queue from the newest batch to the oldest; the arrival-time test ends
      the walk (older batches arrived earlier still), the other tests skip to the next older batch.
  S2  u_b is the utility of the first request that was put into the batch.
  S3  Alg. 2 sorts the queue by d_b ascending, stably.
  S4  DP index l_b = 0 means "batch b is not executed"; l_b = 1..N_gamma selects L^(gamma)[l_b - 1].
      Row 0 of the tables is the state before the first batch (utility 0, clock T).
  S5  the listing writes the processing time once per request and once per batch; it is the
      batch's estimated processing time in both places.
  S6  Profile(B_b, gamma): time = sum over tasks of (requests of the task in the batch) x (profiled
      per-sample latency of the task at gamma), tasks in ascending order; utility = sum over the
      batch's requests, in arrival order, of u_r x (profiled accuracy of r's task at gamma).
  S7  f(q) is a table of (largest request rate, index into L^(gamma)) rows in ascending rate order
      (the paper's Table I); q takes the first row whose largest rate is >= q, so a rate in a gap
      between two printed ranges takes the row above it; a rate above the last row maps to the
      smallest gamma of the list.
  S8  ties: strict comparisons as printed (the first candidate reaching a value keeps it); the final
      arg max takes the lowest index.

  S9  Alg. 2's tables start at dp = 0, S = 1, and a candidate is recorded only when strictly larger
      than the entry.  Taken literally, a state whose best accumulated utility is exactly 0 (all
      earlier batches skipped, or zero-utility requests) keeps S = 1 and C = T, which names a
      predecessor that may be infeasible and loses the clock; the backtracking would then execute a
      batch that cannot meet its deadline, against what the text says J and C are for.  Here the
      initial 0 means "no candidate yet": the first feasible candidate of a state is always
      recorded, later ones only when strictly larger.  Identical to the listing whenever the
      accumulated utility of a state is positive.

Pins (tests/test_sched_pins.py): hand-worked queues for every branch of Alg. 1; Alg. 3 on a
hand-worked queue; Alg. 2 against exhaustive enumeration of all assignments on small queues
(equal to the optimum whenever the deadlines do not bind, never above it, always feasible), and
its reported utility against a replay of the returned plan.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple


@dataclass
class Query:
    s: float          # arrival time
    l: float          # latency requirement
    u: float          # utility
    task: int = 0

    @property
    def d(self) -> float:
        return self.s + self.l


@dataclass
class Batch:
    queries: List[Query] = field(default_factory=list)
    gamma: Optional[int] = None        # index into the selection list, None = not executed / not decided

    @property
    def s(self) -> float:
        return min(q.s for q in self.queries)

    @property
    def d(self) -> float:
        return min(q.d for q in self.queries)

    @property
    def u(self) -> float:
        return self.queries[0].u


# ------------------------------------------------------------------------------- Alg. 1
def add_query(B: List[Batch], r: Query, delta: float, epsilon: int, eta: float, mu: float) -> int:
    """Sec. III-C, Alg. 1: put request r into an existing batch or open a new one.  Returns the index
    of the batch that took it."""
    for b in range(len(B) - 1, -1, -1):
        if B[b].s + delta < r.s:               # arrival time: the batch has waited too long
            break
        elif len(B[b].queries) >= epsilon:     # batch size
            continue
        elif abs(B[b].d - r.d) > eta:          # finish time
            continue
        elif abs(B[b].u - r.u) > mu:           # utility
            continue
        B[b].queries.append(r)
        return b
    B.append(Batch([r]))
    return len(B) - 1


# ------------------------------------------------------------------------------- profile
def profile(batch: Batch, g: int, latency: Sequence[Sequence[float]], accuracy: Sequence[Sequence[float]]):
    """S6.  latency[task][g], accuracy[task][g] are the profiled per-sample latency and accuracy of a
    task at selection-list index g.  Returns (estimated processing time, estimated utility)."""
    n_tasks = len(latency)
    counts = [0] * n_tasks
    for q in batch.queries:
        counts[q.task] += 1
    t = 0.0
    for task in range(n_tasks):
        t += counts[task] * latency[task][g]
    U = 0.0
    for q in batch.queries:
        U += q.u * accuracy[q.task][g]
    return t, U


def rate_table_from_latency(gammas: Sequence[int], latency: Sequence[Sequence[float]]) -> List[Tuple[float, int]]:
    """The projection f of Alg. 3 built from a latency profile (Sec. III-D; Table I is the paper's own
    instance): the gammas from the largest down; a gamma serves every rate up to its throughput
    1 / (mean per-sample latency over the tasks); a gamma that is no faster than the row before it, and
    the smallest gamma (what rates beyond the table get), have no row."""
    n_tasks = len(latency)
    order = sorted(range(len(gammas)), key=lambda i: -gammas[i])
    rows: List[Tuple[float, int]] = []
    for gi in order[:-1]:
        total = 0.0
        for k in range(n_tasks):
            total += latency[k][gi]
        thr = 1.0 / (total / n_tasks)
        if not rows or thr > rows[-1][0]:
            rows.append((thr, gi))
    return rows


def f_of_rate(q: float, table: Sequence[Tuple[float, int]], smallest: int) -> int:
    """S7: selection-list index for request rate q."""
    for q_max, g in table:
        if q <= q_max:
            return g
    return smallest


# ------------------------------------------------------------------------------- Alg. 3
def manually_allocate(B: List[Batch], T: float, gammas: Sequence[int], q: float, f_table, kappa: float,
                      latency, accuracy) -> None:
    """Sec. III-D, Alg. 3: gamma from the request rate, the smallest gamma for a batch that would miss
    its deadline, the largest for a batch of high average utility; the clock advances by each batch's
    estimated time."""
    g_min = min(range(len(gammas)), key=lambda i: gammas[i])
    g_max = max(range(len(gammas)), key=lambda i: gammas[i])
    g = f_of_rate(q, f_table, g_min)
    for b in B:
        t, _ = profile(b, g, latency, accuracy)
        mean_u = sum(x.u for x in b.queries) / len(b.queries)
        if T + t >= b.d:
            b.gamma = g_min
        elif mean_u > kappa:
            b.gamma = g_max
        else:
            b.gamma = g
        t, _ = profile(b, b.gamma, latency, accuracy)
        T = T + t


# ------------------------------------------------------------------------------- Alg. 2
def allocate(B: List[Batch], T: float, gammas: Sequence[int], q: float, beta: int, initial_stage: bool, f_table,
             kappa: float, latency, accuracy) -> float:
    """Sec. III-D, Alg. 2: sorts the queue by deadline and writes b.gamma for every batch (None = not
    executed).  Returns the planned utility (the dynamic program's best value; NaN on the manual
    path)."""
    B.sort(key=lambda b: b.d)
    NB, NG = len(B), len(gammas)
    if NB <= beta or initial_stage:
        manually_allocate(B, T, gammas, q, f_table, kappa, latency, accuracy)
        return float("nan")
    NEG, POS = -math.inf, math.inf
    dp = [[0.0] * (NG + 1) for _ in range(NB + 1)]
    S = [[1] * (NG + 1) for _ in range(NB + 1)]
    C = [[T] * (NG + 1) for _ in range(NB + 1)]
    J = [[0] * (NG + 1) for _ in range(NB + 1)]
    for b in range(1, NB + 1):
        for lb in range(0, NG + 1):
            for lp in range(0, NG + 1):
                if dp[b - 1][lp] == NEG:
                    continue
                if lb == 0:
                    if J[b][lb] == 0 or dp[b - 1][lp] > dp[b][lb]:          # S9
                        dp[b][lb] = dp[b - 1][lp]
                        S[b][lb] = lp
                        C[b][lb] = C[b - 1][lp]
                        J[b][lb] = 1
                else:
                    t, U = profile(B[b - 1], lb - 1, latency, accuracy)
                    if C[b - 1][lp] + t < B[b - 1].d:
                        u = dp[b - 1][lp] + U
                        first = J[b][lb] == 0                               # S9
                        J[b][lb] = 1
                        if first or u > dp[b][lb]:
                            dp[b][lb] = u
                            S[b][lb] = lp
                            C[b][lb] = C[b - 1][lp] + t
            if lb > 0 and J[b][lb] == 0:
                dp[b][lb] = NEG
                C[b][lb] = POS
    l = max(range(NG + 1), key=lambda i: (dp[NB][i], -i))
    best = dp[NB][l]
    B[NB - 1].gamma = None if l == 0 else l - 1
    for b in range(NB - 1, 0, -1):
        l = S[b + 1][l]
        B[b - 1].gamma = None if l == 0 else l - 1
    return best


def replay(B: Sequence[Batch], T: float, latency, accuracy):
    """Runs the batches in queue order with their assigned gamma: returns (utility earned by batches
    that finish before their deadline, final clock, all executed batches met their deadline)."""
    total, ok = 0.0, True
    for b in B:
        if b.gamma is None:
            continue
        t, U = profile(b, b.gamma, latency, accuracy)
        if T + t < b.d:
            total += U
        else:
            ok = False
        T += t
    return total, T, ok
