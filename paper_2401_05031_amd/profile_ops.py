"""Runs ONE operator of the library a few times on synthetic data, for use under a profiler
(`rocprofv3 --pmc ... -- python3 -m paper_2401_05031_amd.profile_ops attention --n 197`): the kernel and
launch configuration are the ones the encoder uses for that shape.  Prints the mean time per launch
measured with HIP events.

    attention --n N [--batch 64] [--D 768] [--H 12] [--size-bias]
    linear    --M M --N N --K K [--epilogue 0|1|2] [--kernel ID]      (ID as in otas_linear_kernel, 0 = the library's choice)
    clock     --M M --N N --K K [--kernel ID] [--zero-data]           (the linear product back to back with the library's
                                                                       shader-clock probe running beside it)
"""
from __future__ import annotations

import argparse

import numpy as np


def main(argv=None) -> None:
    import torch
    from . import OTAS_BF16, OTAS_FLAG_SIZE_BIAS, Context
    ap = argparse.ArgumentParser()
    ap.add_argument("op", choices=["attention", "linear", "clock"])
    ap.add_argument("--n", type=int, default=197)
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--D", type=int, default=768)
    ap.add_argument("--H", type=int, default=12)
    ap.add_argument("--size-bias", action="store_true")
    ap.add_argument("--M", type=int, default=12608)
    ap.add_argument("--N", type=int, default=2304)
    ap.add_argument("--K", type=int, default=768)
    ap.add_argument("--epilogue", type=int, default=0)
    ap.add_argument("--kernel", type=int, default=0)
    ap.add_argument("--iters", type=int, default=3)
    ap.add_argument("--zero-data", action="store_true", help="all-zero operands (clock: the matrix cores then toggle no bits)")
    a = ap.parse_args(argv)
    dev, bf = "cuda", torch.bfloat16
    g = torch.Generator(device="cpu").manual_seed(0)
    D, F = a.D, 4 * a.D
    z = lambda *s: torch.zeros(s, dtype=bf, device=dev)
    layer = {"ln1_g": z(D), "ln1_b": z(D), "w_qkv": z(3 * D, D), "b_qkv": z(3 * D), "w_proj": z(D, D), "b_proj": z(D),
             "ln2_g": z(D), "ln2_b": z(D), "w_fc1": z(F, D), "b_fc1": z(F), "w_fc2": z(D, F), "b_fc2": z(D)}
    ctx = Context(1, D, a.H, F, OTAS_BF16, 1e-6, 1, [layer])
    if a.op == "attention":
        T = a.batch * a.n
        qkv = torch.randn((T, 3 * D), generator=g).to(dev).to(bf)
        sizes = torch.ones(T, dtype=torch.int32, device=dev)
        out = torch.empty((T, D), dtype=bf, device=dev)
        off = np.arange(a.batch + 1, dtype=np.int32) * a.n
        run = lambda: ctx.otas_attention(qkv, sizes, off, OTAS_FLAG_SIZE_BIAS if a.size_bias else 0, out)
        what = f"attention batch {a.batch} n {a.n} D {D} H {a.H}"
    else:
        x = torch.randn((a.M, a.K), generator=g).to(dev).to(bf)
        w = (0.03 * torch.randn((a.N, a.K), generator=g)).to(dev).to(bf)
        if a.zero_data:
            x.zero_(), w.zero_()
        b = torch.zeros(a.N, dtype=bf, device=dev)
        res = torch.zeros((a.M, a.N), dtype=torch.float32, device=dev) if a.epilogue == 2 else None
        y = torch.empty((a.M, a.N), dtype=torch.float32 if a.epilogue == 2 else bf, device=dev)
        run = lambda: ctx.otas_linear_kernel(a.kernel, x, w, b, res, a.M, a.N, a.K, a.epilogue, y)
        what = f"linear {a.M} x {a.N} x {a.K} epilogue {a.epilogue} kernel {a.kernel or ctx.otas_linear_choice(a.M, a.N, a.K, a.epilogue)}"
    run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if a.op == "clock":
        ctx.otas_clock_probe_start(400)
        idle = float(np.median(ctx.otas_clock_probe_read()[40:]))
        e0.record()
        for _ in range(a.iters):
            run()
        e1.record()
        e1.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / a.iters
        ctx.otas_clock_probe_start(int(max(64, min(60000, 0.45 * a.iters * us / 13.55))))
    e0.record()
    for _ in range(a.iters):
        run()
    e1.record()
    e1.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / a.iters
    print(f"{what}{' zero data' if a.zero_data else ''}: {us:.1f} us per launch over {a.iters} launches"
          + (f", {2.0 * a.M * a.N * a.K / us / 1e6:.1f} TFLOP/s" if a.op != "attention" else ""))
    if a.op == "clock":
        mhz = np.asarray(ctx.otas_clock_probe_read())
        mhz = mhz[len(mhz) // 10:]
        print(f"shader clock: idle {idle:.0f} MHz; beside the launches median {np.median(mhz):.0f} MHz, "
              f"10th / 90th percentile {np.percentile(mhz, 10):.0f} / {np.percentile(mhz, 90):.0f} MHz over {len(mhz)} samples")
    ctx.close()


if __name__ == "__main__":
    main()
