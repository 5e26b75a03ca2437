#!/usr/bin/env python3
"""Throughput of the token-adapted encoder on one MI355X.

A step = one pass of the whole hot path over one synthetic batch: otas_prompt_prepend followed by
otas_encoder_forward (LayerNorm, QKV GEMM, attention, projection, merge metric / plan / apply,
LayerNorm, MLP GEMMs, for every layer).  Inputs and weights are resident in HBM before the timed
region.  Prints ONE JSON line: images/s of the headline workload, per-strategy images/s, the
roofline figures of the dominant kernel (the bf16 MFMA GEMM) and of the other kernels, measured
with HIP events through the library's per-launch timing, and the CPU oracle timed on a bounded
sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import otas_synth as synth  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
BASELINE_METRIC = "images/sec per (prompts, r) strategy, ViT-B/16 batch 64 bf16; merge-kernel HBM GB/s"


def algorithmic_work(cfg, lengths0, r, otas):
    """Per-kind algorithmic FLOPs / bytes of ONE forward, from the host-known length schedule."""
    D, H, F, L = cfg.D, cfg.H, cfg.F, cfg.L
    e = 4 if cfg.dtype == "f32" else 2
    sched = np.array([otas.otas_schedule(int(n), 0, int(rr), cfg.n_lead, L) for n, rr in zip(lengths0, r)])  # [B, L+1]
    T = sched.sum(axis=0)
    w = {"gemm_qkv": 0.0, "gemm_proj": 0.0, "gemm_fc1": 0.0, "gemm_fc2": 0.0, "attention": 0.0,
         "merge_apply_bytes": 0.0, "layer_norm_bytes": 0.0, "merge_layers": 0}
    for l in range(L):
        w["gemm_qkv"] += 2.0 * T[l] * D * 3 * D
        w["gemm_proj"] += 2.0 * T[l] * D * D
        w["gemm_fc1"] += 2.0 * T[l + 1] * D * F
        w["gemm_fc2"] += 2.0 * T[l + 1] * D * F
        w["attention"] += float(np.sum(4.0 * sched[:, l].astype(np.float64) ** 2 * D))
        w["layer_norm_bytes"] += T[l] * D * (4.0 + e)                # LN1: float residual row in, operand row out
        if T[l + 1] != T[l]:
            # merge-apply fused with LN2: float rows in and out, a size and a list entry per row, operand row out
            w["merge_apply_bytes"] += (T[l] + T[l + 1]) * (D * 4.0 + 8.0) + T[l + 1] * D * e
        else:
            w["layer_norm_bytes"] += T[l + 1] * D * (4.0 + e)        # LN2 on its own
            w["merge_layers"] += 1
    w["T"] = T.tolist()
    return w


def run_strategy(name, steps, warmup, timing_steps):
    import torch
    import paper_2401_05031_amd as otas

    cfg = synth.config(name)
    ctx = otas.Context.from_host_weights(cfg.L, cfg.D, cfg.H, cfg.F,
                                         otas.OTAS_F32 if cfg.dtype == "f32" else otas.OTAS_BF16,
                                         cfg.ln_eps, cfg.n_lead, synth.all_weights(cfg))
    toks, prm, P, R = synth.batch(cfg)
    D = cfg.D
    tok_packed, tok_off = synth.pack(toks, D)
    prm_packed, prm_off = synth.pack(prm, D)
    t_tok = torch.from_numpy(tok_packed).to("cuda").to(ctx.torch_dtype)
    t_prm = torch.from_numpy(prm_packed).to("cuda").to(ctx.torch_dtype) if prm_packed.shape[0] else None
    T0 = int(tok_off[-1] + prm_off[-1])
    x0 = torch.empty((T0, D), dtype=ctx.torch_dtype, device="cuda")
    lengths0 = np.diff(tok_off) + np.diff(prm_off)
    reff, _ = ctx.trace_layout(lengths0, R)
    T_out = int(T0 - reff.sum())
    ws = torch.empty(ctx.otas_workspace_bytes(cfg.B, T0), dtype=torch.uint8, device="cuda")
    x_out = torch.empty((T_out, D), dtype=torch.float32, device="cuda")
    sizes_out = torch.empty(T_out, dtype=torch.int32, device="cuda")

    def step():
        off = ctx.otas_prompt_prepend(t_tok, tok_off, t_prm, prm_off, x0)
        ctx.otas_encoder_forward(x0, off, R, 0, ws, x_out, sizes_out)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = dt / steps * 1e3

    # per-kernel durations: the same steps again with an event pair around every launch
    ctx.otas_timing_enable(True)
    for _ in range(timing_steps):
        step()
    kt = ctx.otas_timing_read()
    ev_overhead_us = ctx.otas_timing_overhead_ms() * 1e3
    ctx.otas_timing_enable(False)
    per_step = {k: (v[0] / timing_steps, v[1] // timing_steps) for k, v in kt.items()}
    work = algorithmic_work(cfg, lengths0, R, otas)
    assert torch.isfinite(x_out.float()).all()
    ctx.close()
    return {"name": name, "cfg": cfg, "ms": ms, "img_s": cfg.B / (ms * 1e-3), "kernels": per_step, "work": work,
            "ev_overhead_us": ev_overhead_us}


def measured_traffic(workload):
    """Per-launch HBM bytes per kernel family measured offline with rocprofv3 --pmc (see
    paper_2401_05031_amd/traffic.py); None for workloads that were not measured."""
    path = os.path.join(ROOT, "paper_2401_05031_amd", "hbm_traffic.json")
    try:
        d = json.load(open(path))
    except OSError:
        return {}
    return {k: v["bytes"] for k, v in d["families"].items()} if d.get("workload") == workload else {}


def rooflines(res):
    k, w = res["kernels"], res["work"]
    traffic = measured_traffic(res["name"])
    gemm_ms = sum(k[n][0] for n in ("gemm_qkv", "gemm_proj", "gemm_fc1", "gemm_fc2"))
    gemm_launches = sum(k[n][1] for n in ("gemm_qkv", "gemm_proj", "gemm_fc1", "gemm_fc2"))
    gemm_flops = sum(w[n] for n in ("gemm_qkv", "gemm_proj", "gemm_fc1", "gemm_fc2"))
    out = {}
    ach = gemm_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    out["gemm"] = {"bound": "mfma", "achieved": round(ach, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                   "frac": round(ach / PEAK_BF16_TFLOPS, 4), "traffic": traffic.get("gemm"),
                   "launches_per_step": gemm_launches, "avg_launch_us": round(gemm_ms * 1e3 / max(gemm_launches, 1), 2),
                   "flops_per_launch": gemm_flops / max(gemm_launches, 1)}
    for n in ("gemm_qkv", "gemm_proj", "gemm_fc1", "gemm_fc2"):
        if k[n][0] > 0:
            a = w[n] / (k[n][0] * 1e-3) / 1e12
            out[n] = {"bound": "mfma", "achieved": round(a, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                      "frac": round(a / PEAK_BF16_TFLOPS, 4), "avg_launch_us": round(k[n][0] * 1e3 / max(k[n][1], 1), 2)}
    if k["attention"][0] > 0:
        a = w["attention"] / (k["attention"][0] * 1e-3) / 1e12
        out["attention"] = {"bound": "mfma", "achieved": round(a, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                            "frac": round(a / PEAK_BF16_TFLOPS, 4), "traffic": traffic.get("attention"),
                            "avg_launch_us": round(k["attention"][0] * 1e3 / max(k["attention"][1], 1), 2)}
    if k["merge_apply"][0] > 0:
        a = w["merge_apply_bytes"] / (k["merge_apply"][0] * 1e-3) / 1e9
        out["merge_apply"] = {"bound": "hbm", "achieved": round(a, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                              "frac": round(a / PEAK_HBM_GBS, 4), "traffic": traffic.get("merge_apply"),
                              "algorithmic_bytes_per_launch": round(w["merge_apply_bytes"] / max(k["merge_apply"][1], 1)),
                              "avg_launch_us": round(k["merge_apply"][0] * 1e3 / max(k["merge_apply"][1], 1), 2)}
    if k["layer_norm"][0] > 0:
        a = w["layer_norm_bytes"] / (k["layer_norm"][0] * 1e-3) / 1e9
        out["layer_norm"] = {"bound": "hbm", "achieved": round(a, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                             "frac": round(a / PEAK_HBM_GBS, 4), "traffic": traffic.get("layer_norm"),
                             "avg_launch_us": round(k["layer_norm"][0] * 1e3 / max(k["layer_norm"][1], 1), 2)}
    for n in ("merge_plan", "prompt_prepend"):
        if k[n][1] > 0:
            out[n] = {"avg_launch_us": round(k[n][0] * 1e3 / k[n][1], 2), "launches_per_step": k[n][1]}
    out["kernel_ms_per_step"] = {n: round(v[0], 4) for n, v in k.items()}
    out["event_pair_overhead_us_subtracted"] = round(res["ev_overhead_us"], 2)
    return out


def cpu_baseline(name, n_queries):
    """The oracle, as it stands, on the host cores over a bounded sample of the same workload."""
    from oracle import otas_oracle as orc
    cfg = synth.config(name)
    layers = synth.all_weights(cfg)
    toks, prm, P, R = synth.batch(cfg, list(range(n_queries)))
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    storage = "bf16" if cfg.dtype == "bf16" else "f64"
    t0 = time.perf_counter()
    for q in range(n_queries):
        x0, _ = orc.prompt_prepend(toks[q], prm[q], cfg.n_lead)
        orc.encoder_forward_query(x0, layers, R[q], H=cfg.H, ln_eps=cfg.ln_eps, n_lead=cfg.n_lead, storage=storage)
    dt = time.perf_counter() - t0
    return {"value": round(n_queries / dt, 3), "unit": "images/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{n_queries} of {cfg.B} queries of {name} (float64 NumPy oracle with bf16 storage rounding), "
                      f"{dt:.1f} s; host has {len(os.sched_getaffinity(0))} usable cores"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="vitb_r16", choices=list(synth.CONFIG_NAMES))
    ap.add_argument("--others", default="vitb_plain,vitb_p10_r8", help="further strategies reported per strategy")
    ap.add_argument("--cpu-queries", type=int, default=12)
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run one plain device copy of 256 MiB (torch) so that a rocprofv3 --pmc run of this "
                         "command holds a kernel of known HBM traffic to scale FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (queries are independent, so more GPUs would be plain data "
              "parallelism with no collective); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)

    if args.calibrate:
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)                      # 256 MiB read + 256 MiB written
        torch.cuda.synchronize()
        del a, b
    head = run_strategy(args.workload, args.steps, args.warmup, timing_steps=max(3, min(10, args.steps)))
    per_strategy = {}
    all_res = [head]
    for n in [s for s in args.others.split(",") if s and s != args.workload]:
        all_res.append(run_strategy(n, max(5, args.steps // 2), args.warmup, timing_steps=3))
    for r in all_res:
        P, R = r["cfg"].strategies[0]
        mixed = len(set(r["cfg"].strategies)) > 1
        rf = rooflines(r)
        per_strategy[r["name"]] = {
            "strategy": "mixed" if mixed else {"prompts": P, "r": R},
            "images_per_s": round(r["img_s"], 1), "ms_per_step": round(r["ms"], 4),
            "gemm_tflops": rf["gemm"]["achieved"],
            "merge_apply_gbs": rf.get("merge_apply", {}).get("achieved"),
            "attention_tflops": rf.get("attention", {}).get("achieved"),
        }
    rf = rooflines(head)
    cfg = head["cfg"]
    out = {
        "metric": BASELINE_METRIC, "value": round(head["img_s"], 1), "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(head["ms"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: L={cfg.L} D={cfg.D} H={cfg.H} F={cfg.F}, batch {cfg.B} x {cfg.n0} tokens, "
                               f"strategy (P, r) = {'mixed' if len(set(cfg.strategies)) > 1 else cfg.strategies[0]}",
                   "global_batch": cfg.B, "seq_len": cfg.n0, "parallelism": "single GPU"},
        "roofline": {k: rf["gemm"][k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic")},
        "rooflines": rf,
        "per_strategy": per_strategy,
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(args.workload, args.cpu_queries)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
