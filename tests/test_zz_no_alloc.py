"""otas_token_merge_static (the entry point that allocates nothing: its merge lists live in a static
device array of the library) against otas_token_merge on the same inputs: same kernels, so tokens,
sizes, offsets and the edge trace must be identical bit for bit.  Two calls in a row on one context,
the second with a smaller batch, so that whatever the first call left in the shared array would show
if the second read it; then the size limits."""
import numpy as np
import pytest

import otas_synth as synth
from tests import harness as hz

pytestmark = pytest.mark.gpu


def _both(torch, ctx, cfg, ns, rs, dm, seed, sizes_hi):
    rng = np.random.default_rng(seed)
    rnd = synth.round_to_bf16 if cfg.dtype == "bf16" else (lambda a: a.astype(np.float32))
    xs = [rnd(rng.standard_normal((n, cfg.D)).astype(np.float32)) for n in ns]
    ms = [rnd(rng.standard_normal((n, dm)).astype(np.float32)) for n in ns]
    szs = [rng.integers(1, sizes_hi + 1, n).astype(np.int32) for n in ns]
    xp, off = synth.pack(xs, cfg.D)
    mp, _ = synth.pack(ms, dm)
    T = int(off[-1])
    dt = ctx.torch_dtype
    x_d = torch.from_numpy(xp).to("cuda").to(dt)
    m_d = torch.from_numpy(mp).to("cuda").to(dt)
    s_d = torch.from_numpy(np.concatenate(szs)).to("cuda") if sizes_hi > 1 else None
    n_tr = max(sum(min(r, (n - cfg.n_lead) // 2) for n, r in zip(ns, rs)), 1)

    def outputs():
        return (torch.full((T, cfg.D), float("nan"), dtype=dt, device="cuda"),
                torch.full((T,), -7, dtype=torch.int32, device="cuda"),
                torch.full((n_tr,), -1, dtype=torch.int32, device="cuda"),
                torch.full((n_tr,), -1, dtype=torch.int32, device="cuda"))

    ws = torch.empty(ctx.otas_merge_workspace_bytes(len(ns), T), dtype=torch.uint8, device="cuda")
    xa, sa, ta, da = outputs()
    off_a = ctx.otas_token_merge(x_d, m_d, dm, s_d, off, rs, ws, xa, sa, ta, da)
    xb, sb, tb, db = outputs()                       # allocated BEFORE the call under test
    torch.cuda.synchronize()
    off_b = ctx.otas_token_merge_static(x_d, m_d, dm, s_d, off, rs, xb, sb, tb, db)
    torch.cuda.synchronize()
    assert off_a.tolist() == off_b.tolist()
    T_out = int(off_a[-1])
    assert T_out < T or all(r == 0 for r in rs)
    assert torch.equal(xa[:T_out].view(torch.int16 if dt == torch.bfloat16 else torch.int32),
                       xb[:T_out].view(torch.int16 if dt == torch.bfloat16 else torch.int32))
    assert torch.equal(sa[:T_out], sb[:T_out]) and int(sb[:T_out].min()) >= 1
    assert torch.equal(ta, tb) and torch.equal(da, db)
    return T_out


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_static_scratch_merge_equals_workspace_merge_twice_in_a_row(dtype):
    import torch
    assert torch.cuda.is_available()
    import paper_2401_05031_amd as otas
    cfg = synth.config("tiny")
    cfg.dtype = dtype
    ctx, _ = hz.make_context(cfg)
    # first call: a ragged batch spanning many rows; second call: fewer and shorter queries, so it
    # uses a prefix of the lists the first call wrote
    big_ns = [201, 197, 2, 3, 1, 64, 267, 130, 5] * 3
    big_rs = [8, 16, 5, 1, 4, 0, 100, 24, 2] * 3
    t1 = _both(torch, ctx, cfg, big_ns, big_rs, 64, seed=21, sizes_hi=4)
    t2 = _both(torch, ctx, cfg, [150, 33, 197], [20, 3, 16], 80, seed=22, sizes_hi=1)
    assert t2 < t1
    # limits: too many rows or queries are refused before any launch
    n = 1024
    B = otas.binding.OTAS_STATIC_MERGE_MAX_ROWS // n + 1
    x = torch.zeros((B * n, cfg.D), dtype=ctx.torch_dtype, device="cuda")
    m = torch.zeros((B * n, 64), dtype=ctx.torch_dtype, device="cuda")
    xo = torch.empty_like(x)
    so = torch.empty(B * n, dtype=torch.int32, device="cuda")
    with pytest.raises(otas.OtasError) as e:
        ctx.otas_token_merge_static(x, m, 64, None, np.arange(B + 1) * n, [0] * B, xo, so)
    assert e.value.status == 3
    Bq = otas.binding.OTAS_STATIC_MERGE_MAX_QUERIES + 1
    with pytest.raises(otas.OtasError) as e:
        ctx.otas_token_merge_static(x, m, 64, None, np.arange(Bq + 1) * 2, [0] * Bq, xo, so)
    assert e.value.status == 3
    # a query too long for the plan kernel's LDS would need workspace for its metric rows: refused here
    # (otas_token_merge takes it), with or without merging in it
    with pytest.raises(otas.OtasError) as e:
        ctx.otas_token_merge_static(x[:700], m[:700], 64, None, [0, 700], [4], xo[:700], so[:700])
    assert e.value.status == 5
    # and a third, ordinary call still works after the refused ones
    _both(torch, ctx, cfg, [197, 197], [16, 8], 64, seed=23, sizes_hi=2)
    ctx.close()
