"""The serving loop around the library: requests arrive, adaptive batching (Sec. III-C, Alg. 1) groups
them, token adaptation (Sec. III-D, Alg. 2 / Alg. 3) gives every queued batch a gamma, and the execution
engine runs the batch at the head of the queue with that gamma (Fig. 3, workflow; Sec. IV, interfaces).

The paper prints no listing for the loop itself; this one makes the following choices:
  * one engine, batches run one after another; whenever the engine is free and the queue is not empty,
    all requests that have arrived are admitted, the arriving rate q is the number of arrivals in the
    last `rate_window` seconds divided by that window, and one allocation pass runs over the whole queue;
  * the first batch in deadline order that the pass decided to execute runs next, to completion;
  * a batch the pass skipped stays queued for the next pass unless even the smallest gamma could no longer
    finish it in time, in which case it is given up; when nothing is runnable the clock moves to the next
    arrival, or, with no arrivals left, the remaining batches are given up;
  * a request earns u_r times the profiled accuracy of its task at the batch's gamma when its batch
    finishes before the request's own deadline (alpha_r of Eq. 3), nothing otherwise.
The clock is virtual: it advances by what the engine reports for each batch, so a trace replays as fast
as the engine runs.  With `GpuEngine` every batch really runs through otas_encoder_forward and
otas_task_heads and the clock advances by the measured time; `ProfileEngine` advances it by the profile
table's estimate (no GPU needed: a simulation of the same loop).

The scheduler argument is any object with the otas_sched_* methods of binding.Scheduler.
"""
from __future__ import annotations

import time
from typing import Dict, List, Sequence, Tuple

import numpy as np

from .binding import OTAS_BF16, Context, Scheduler, otas_sched_rate_table  # noqa: F401


def gamma_to_strategy(gamma: int) -> Tuple[int, int]:
    """(P, r) of a gamma value: gamma > 0 adds gamma prompt tokens, gamma < 0 merges -gamma tokens per
    layer, 0 is the plain model (Sec. III-D, definition of gamma_b)."""
    return (gamma, 0) if gamma > 0 else (0, -gamma)


class ProfileEngine:
    """Engine of the simulation: a batch takes exactly what the profile table predicts."""

    def __init__(self, latency):
        self.latency = np.asarray(latency, dtype=np.float64)

    def run(self, tasks: Sequence[int], gamma_index: int, gamma: int) -> float:
        t = 0.0
        counts = np.bincount(np.asarray(tasks, dtype=np.int64), minlength=self.latency.shape[0])
        for k in range(self.latency.shape[0]):
            t += int(counts[k]) * self.latency[k][gamma_index]
        return t


class GpuEngine:
    """Runs every batch on the GPU: prompt prepend, the token-adapted encoder, final norm and per-task
    heads.  Token embeddings come from a resident pool of `pool` synthetic images' tokens (request i uses
    slot i mod pool); per-task prompt pools hold max(gammas) rows.  run() returns the measured wall-clock
    seconds of the batch, host launch cost included."""

    def __init__(self, ctx: Context, n_tokens: int, task_classes: Sequence[int], max_prompts: int, pool: int = 64,
                 seed: int = 0):
        import torch
        self.torch = torch
        self.ctx, self.n, self.pool = ctx, n_tokens, pool
        D = ctx.D
        g = torch.Generator(device="cpu").manual_seed(seed)
        dt = ctx.torch_dtype
        self.tokens = torch.randn((pool * n_tokens, D), generator=g).to("cuda").to(dt)
        # the prompt repository: task k's trained prompts are rows k * max_prompts .. of one device tensor
        self.prompt_pool = (0.02 * torch.randn((len(task_classes) * max_prompts, D), generator=g)).to("cuda").to(dt)
        self.heads = [((0.02 * torch.randn((k, D), generator=g)).to("cuda").to(dt).contiguous(),
                       torch.zeros(k).to("cuda").to(dt)) for k in task_classes]
        self.lnf_g = torch.ones(D).to("cuda").to(dt)
        self.lnf_b = torch.zeros(D).to("cuda").to(dt)
        self.max_prompts = max_prompts
        T_max = pool * (n_tokens + max_prompts)
        self.x0 = torch.empty((T_max, D), dtype=dt, device="cuda")
        self.x_out = torch.empty((T_max, D), dtype=torch.float32, device="cuda")
        self.sizes_out = torch.empty(T_max, dtype=torch.int32, device="cuda")
        self.ws = torch.empty(ctx.otas_workspace_bytes(pool, T_max), dtype=torch.uint8, device="cuda")
        self.logits = torch.empty((pool, max(task_classes)), dtype=torch.float32, device="cuda")

    def run(self, tasks: Sequence[int], gamma_index: int, gamma: int) -> float:
        torch = self.torch
        B = len(tasks)
        if B > self.pool:
            raise ValueError(f"batch of {B} exceeds the engine's pool of {self.pool}")
        P, r = gamma_to_strategy(gamma)
        if P > self.max_prompts:
            raise ValueError("gamma beyond the prompt pool")
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        tok_off = np.arange(B + 1, dtype=np.int32) * self.n
        first = [k * self.max_prompts for k in tasks]           # every query takes the first P rows of its task
        off = self.ctx.otas_prompt_prepend_pool(self.tokens[:B * self.n], tok_off, self.prompt_pool, first, [P] * B,
                                                self.x0)
        out_off = self.ctx.otas_encoder_forward(self.x0, off, [r] * B, 0, self.ws, self.x_out, self.sizes_out)
        self.ctx.otas_task_heads(self.x_out, out_off, list(tasks), self.heads, self.lnf_g, self.lnf_b, self.logits[:B])
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def measure_profile(self, gammas: Sequence[int], n_tasks: int, batch: int, repeats: int = 5) -> np.ndarray:
        """[n_tasks][len(gammas)] per-sample latency in seconds: the median batch time at `batch` requests
        divided by the batch size (Sec. III-D: sample-level inference latency per task and gamma)."""
        lat = np.zeros((n_tasks, len(gammas)))
        for k in range(n_tasks):
            for gi, g in enumerate(gammas):
                self.run([k] * batch, gi, g)
                ts = sorted(self.run([k] * batch, gi, g) for _ in range(repeats))
                lat[k, gi] = ts[len(ts) // 2] / batch
        return lat


def rate_table_from_latency(gammas: Sequence[int], latency) -> List[Tuple[float, int]]:
    """The projection f of Alg. 3 profiled from throughput: otas_sched_rate_table of the library."""
    return otas_sched_rate_table(gammas, latency)


def replay_trace(sched, trace: Sequence[Tuple[float, float, float, int]], engine, accuracy, initial_stage: float = 2.0,
                 rate_window: float = 1.0, log: bool = False) -> Dict:
    """Replays rows (s_r, l_r, u_r, task) in arrival order through the loop described in the module
    docstring.  Returns utility, counts and, with log=True, one record per engine run and give-up."""
    acc = np.asarray(accuracy, dtype=np.float64)
    gammas = list(sched.gammas)
    g_small = min(range(len(gammas)), key=lambda i: gammas[i])
    arrivals = np.asarray([row[0] for row in trace], dtype=np.float64)
    n = len(trace)
    T, i = 0.0, 0
    res = {"utility": 0.0, "offered_utility": float(sum(row[2] for row in trace)), "served": 0, "late": 0,
           "given_up": 0, "batches": 0, "busy": 0.0, "allocate_seconds": 0.0, "allocate_calls": 0, "gamma_batches": {g: 0 for g in gammas}, "log": []}
    while i < n or sched.otas_sched_num_batches() > 0:
        while i < n and arrivals[i] <= T:
            s_r, l_r, u_r, task = trace[i]
            sched.otas_sched_add_query(i, s_r, l_r, u_r, task)
            i += 1
        nb = sched.otas_sched_num_batches()
        if nb == 0:
            T = float(arrivals[i])
            continue
        lo = int(np.searchsorted(arrivals, T - rate_window, side="right"))
        hi = int(np.searchsorted(arrivals, T, side="right"))
        q = (hi - lo) / rate_window
        t_host = time.perf_counter()
        sched.otas_sched_allocate(T, q, T < initial_stage)
        res["allocate_seconds"] += time.perf_counter() - t_host
        res["allocate_calls"] += 1
        pick = -1
        hopeless = []
        for b in range(nb):
            info = sched.otas_sched_batch_info(b)
            if info["gamma_index"] >= 0:
                pick = b
                break
            t_min, _ = sched.otas_sched_estimate(b, g_small)
            if T + t_min >= info["d_b"]:
                hopeless.append(b)
        if pick < 0 and not hopeless:
            if i < n:
                T = max(T, float(arrivals[i]))
                continue
            hopeless = list(range(nb))
        if pick >= 0:
            gi = sched.otas_sched_batch_info(pick)["gamma_index"]
            ids, tasks = sched.otas_sched_batch_queries(pick)
            dt = engine.run(tasks, gi, gammas[gi])
            T_end = T + dt
            for rid, task in zip(ids, tasks):
                s_r, l_r, u_r, _ = trace[rid]
                if T_end < s_r + l_r:
                    res["utility"] += u_r * acc[task][gi]
                    res["served"] += 1
                else:
                    res["late"] += 1
            res["batches"] += 1
            res["busy"] += dt
            res["gamma_batches"][gammas[gi]] += 1
            if log:
                res["log"].append(("run", T, tuple(ids), gammas[gi], dt))
            sched.otas_sched_remove(pick)
            hopeless = [b for b in hopeless if b < pick]      # positions before the pick are unchanged
            T = T_end
        for b in reversed(hopeless):
            ids, _ = sched.otas_sched_batch_queries(b)
            res["given_up"] += len(ids)
            if log:
                res["log"].append(("give_up", T, tuple(ids)))
            sched.otas_sched_remove(b)
    res["end_time"] = T
    return res


def main(argv=None) -> None:
    """Profiles the library on this GPU for every gamma of the paper's selection list, then replays a
    synthetic trace (Sec. V workload shape) through the loop with the GPU engine: once with token
    adaptation, once with every batch at gamma = 0.  The trace's clock is compressed so that the plain
    model's measured capacity stands where the paper's machine had it (580 requests / s at gamma = 0,
    Sec. II-C) relative to the 200..700 requests / s load; thresholds given in seconds scale with it.
    Prints one JSON line."""
    import argparse
    import gc
    import json
    import os
    import sys

    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import otas_synth as synth

    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="vitb_plain")
    ap.add_argument("--seconds", type=int, default=60, help="length of the trace on the paper's clock")
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--load", type=float, default=1.0, help="multiplies the trace's request rates")
    args = ap.parse_args(argv)
    cfg = synth.config(args.workload)
    ctx = Context.from_host_weights(cfg.L, cfg.D, cfg.H, cfg.F, OTAS_BF16, cfg.ln_eps, cfg.n_lead,
                                    synth.all_weights(cfg))
    gammas = list(synth.GAMMA_LIST)
    n_tasks = len(synth.TASK_CLASSES)
    eng = GpuEngine(ctx, cfg.n0, synth.TASK_CLASSES, max(gammas), pool=64)
    lat = eng.measure_profile(gammas, n_tasks, batch=64)
    acc = synth.stand_in_accuracy(gammas, n_tasks)
    gc.collect()
    gc.freeze()     # a full collection (tens of ms with torch imported) must not land inside a measured batch
    thr0 = 1.0 / float(lat[:, gammas.index(0)].mean())
    scale = 580.0 / thr0
    trace = synth.poisson_trace(args.seed, args.seconds, 200.0 * args.load, 700.0 * args.load, time_scale=scale)
    kw = dict(delta=0.5 * scale, eta=0.5 * scale)
    out = {"workload": args.workload, "batch": 64, "gammas": gammas,
           "images_per_s": [round(1.0 / float(lat[:, i].mean()), 1) for i in range(len(gammas))],
           "time_scale": scale, "load": args.load, "requests": len(trace)}
    for name, gl in (("adaptive", gammas), ("fixed_gamma_0", [0])):
        idx = [gammas.index(g) for g in gl]
        l2, a2 = lat[:, idx], acc[:, idx]
        sched = Scheduler(gl, l2, a2, rate_table_from_latency(gl, l2), **kw)
        t0 = time.perf_counter()
        r = replay_trace(sched, trace, eng, a2, initial_stage=2.0 * scale, rate_window=1.0 * scale)
        r.pop("log")
        r["wall_seconds"] = time.perf_counter() - t0
        r["gamma_batches"] = {str(k): v for k, v in r["gamma_batches"].items()}
        out[name] = {k: (round(v, 6) if isinstance(v, float) else v) for k, v in r.items()}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
