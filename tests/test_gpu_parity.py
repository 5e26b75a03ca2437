"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Error metric of every value bar: max |got - ref| / max |ref| over a query's output tensor
(harness.rel_err); beside it harness.elem_err, the element-wise relative error with the tensor's rms
as the absolute floor, is asserted against bars of its own.
Bars: f32 -- merge edges and sizes bit-exact, values <= 1e-4.  bf16 -- the target is values <= 2e-2
and < 0.1 % of merge decisions differing; the tests hold the kernels to what they deliver, which is
tighter on values (<= 1e-2) and, for decisions, the 0.1 % bar block by block on identical inputs
(no slack; >= 1000 decisions per case) and the oracle's own noise floor end to end (<= 1.5 % of
decisions, every differing edge within NEAR_TIE), with the oracle rounding at the same storage
points and adopting the GPU's decisions layer by layer."""
import numpy as np
import pytest

import otas_synth as synth
from oracle import otas_oracle as orc
from tests import harness as hz

pytestmark = pytest.mark.gpu

F32_TOL = 1e-4
BF16_TOL = 1e-2                 # the target is 2e-2; measured <= 5.4e-3
BF16_ELEM_TOL = 5e-2            # element-wise, floor = rms of the tensor (harness.elem_err); measured <= 2.6e-2
F32_ELEM_TOL = 1e-5             # measured 4.5e-7
BF16_DECISION_TOL = 1e-3        # block by block, identical inputs
BF16_E2E_DECISION_TOL = 1.5e-2  # end to end, the oracle's own noise floor (tests/test_bf16_noise_floor.py)


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


def _t(torch, a, dt):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda").to(dt).contiguous()


# ------------------------------------------------------------------ whole encoder, f32 config
def test_tiny_f32_encoder_bit_exact_decisions(torch_cuda, lib):
    cfg = synth.config("tiny")
    ctx, layers = hz.make_context(cfg)
    toks, prm, P, R = synth.batch(cfg)
    x0, off = hz.gpu_prepend(ctx, toks, prm)
    assert off.tolist() == [0, 201, 402]
    gpu = hz.gpu_forward(ctx, x0, off, R)
    ref = hz.oracle_forward(cfg, layers, toks, prm, R)
    margins = []
    for q in range(cfg.B):
        assert np.array_equal(gpu["sizes"][q], ref[q]["sizes"])
        for l in range(cfg.L):
            assert np.array_equal(gpu["trace"][q][l][0], ref[q]["trace"][l][0]), (q, l)
            assert np.array_equal(gpu["trace"][q][l][1], ref[q]["trace"][l][1]), (q, l)
            margins.append((ref[q]["margins"][l]["argmax_margin"], ref[q]["margins"][l]["rank_margin"]))
        assert gpu["x"][q].shape == ref[q]["x"].shape == (185, cfg.D)
        assert hz.rel_err(gpu["x"][q], ref[q]["x"]) <= F32_TOL
        assert hz.elem_err(gpu["x"][q], ref[q]["x"]) <= F32_ELEM_TOL
        print("tiny f32 query", q, "rel_err %.2e elem_err %.2e" % (hz.rel_err(gpu["x"][q], ref[q]["x"]),
                                                                  hz.elem_err(gpu["x"][q], ref[q]["x"])))
    print("min decision margins (argmax, rank):", np.min(np.array(margins), axis=0))
    assert gpu["offsets"].tolist() == [0, 185, 370]
    ctx.close()


def test_tiny_f32_size_bias_flag(torch_cuda, lib):
    cfg = synth.config("tiny")
    ctx, layers = hz.make_context(cfg)
    toks, prm, P, R = synth.batch(cfg)
    x0, off = hz.gpu_prepend(ctx, toks, prm)
    gpu = hz.gpu_forward(ctx, x0, off, R, flags=lib.OTAS_FLAG_SIZE_BIAS)
    ref = hz.oracle_forward(cfg, layers, toks, prm, R, size_bias=True)
    plain = hz.oracle_forward(cfg, layers, toks, prm, R)
    for q in range(cfg.B):
        assert np.array_equal(gpu["sizes"][q], ref[q]["sizes"])
        assert hz.rel_err(gpu["x"][q], ref[q]["x"]) <= F32_TOL
        assert hz.rel_err(ref[q]["x"], plain[q]["x"]) > 1e-3      # the flag is not a no-op here
    ctx.close()


def test_gamma_zero_is_plain_encoder_f32(torch_cuda, lib):
    cfg = synth.config("tiny")
    cfg.strategies = [(0, 0), (0, 0)]
    ctx, layers = hz.make_context(cfg)
    toks, prm, P, R = synth.batch(cfg)
    x0, off = hz.gpu_prepend(ctx, toks, prm)
    gpu = hz.gpu_forward(ctx, x0, off, R)
    ref = hz.oracle_forward(cfg, layers, toks, prm, R)
    for q in range(cfg.B):
        assert gpu["sizes"][q].tolist() == [1] * 197
        assert hz.rel_err(gpu["x"][q], ref[q]["x"]) <= F32_TOL
    ctx.close()


# ------------------------------------------------------------------ single steps
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_prompt_prepend_ragged(torch_cuda, lib, dtype):
    torch = torch_cuda
    cfg = synth.config("tiny")
    cfg.dtype = dtype
    ctx, _ = hz.make_context(cfg)
    rng = np.random.default_rng(3)
    ns, Ps = [5, 1, 197, 33, 64], [0, 3, 10, 0, 1]
    rnd = synth.round_to_bf16 if dtype == "bf16" else (lambda a: a.astype(np.float32))
    toks = [rnd(rng.standard_normal((n, cfg.D)).astype(np.float32)) for n in ns]
    prm = [rnd(rng.standard_normal((p, cfg.D)).astype(np.float32)) for p in Ps]
    out, off = hz.gpu_prepend(ctx, toks, prm)
    got = out.to(torch.float32).cpu().numpy()
    assert off.tolist() == np.concatenate([[0], np.cumsum(np.array(ns) + np.array(Ps))]).tolist()
    for q in range(len(ns)):
        ref, _ = orc.prompt_prepend(toks[q], prm[q], cfg.n_lead)
        assert np.array_equal(got[off[q]:off[q + 1]], ref.astype(np.float32))       # a copy: bit-exact
    ctx.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_prompt_prepend_from_a_prompt_pool(torch_cuda, lib, dtype):
    """otas_prompt_prepend_pool: every query takes a row range of one prompt repository (shared ranges,
    empty ranges, the last rows of the pool); bit-exact against the oracle's prepend; ranges outside the
    pool are refused."""
    torch = torch_cuda
    cfg = synth.config("tiny")
    cfg.dtype = dtype
    ctx, _ = hz.make_context(cfg)
    rng = np.random.default_rng(77)
    rnd = synth.round_to_bf16 if dtype == "bf16" else (lambda a: a.astype(np.float32))
    ns = [197, 1, 5, 64, 33, 2]
    pool = rnd(rng.standard_normal((24, cfg.D)).astype(np.float32))
    first = [0, 8, 8, 20, 3, 16]
    count = [8, 4, 4, 4, 0, 8]
    toks = [rnd(rng.standard_normal((n, cfg.D)).astype(np.float32)) for n in ns]
    tp, toff = synth.pack(toks, cfg.D)
    out = torch.full((sum(ns) + sum(count), cfg.D), float("nan"), dtype=ctx.torch_dtype, device="cuda")
    off = ctx.otas_prompt_prepend_pool(_t(torch, tp, ctx.torch_dtype), toff, _t(torch, pool, ctx.torch_dtype), first,
                                       count, out)
    torch.cuda.synchronize()
    got = out.to(torch.float32).cpu().numpy()
    assert off.tolist() == np.concatenate([[0], np.cumsum(np.array(ns) + np.array(count))]).tolist()
    for q in range(len(ns)):
        ref, _ = orc.prompt_prepend(toks[q], pool[first[q]:first[q] + count[q]], cfg.n_lead)
        assert np.array_equal(got[off[q]:off[q + 1]], ref.astype(np.float32))
    for bad_first, bad_count in (([0, 8, 8, 21, 3, 16], count), ([-1, 8, 8, 20, 3, 16], count), (first, [8, 4, -1, 4, 0, 8])):
        with pytest.raises(lib.OtasError) as e:
            ctx.otas_prompt_prepend_pool(_t(torch, tp, ctx.torch_dtype), toff, _t(torch, pool, ctx.torch_dtype),
                                         bad_first, bad_count, out)
        assert e.value.status == 1
    ctx.close()


def _merge_case(torch, ctx, cfg, ns, rs, dm, seed, sizes_hi=1, dup=False):
    rng = np.random.default_rng(seed)
    rnd = synth.round_to_bf16 if cfg.dtype == "bf16" else (lambda a: a.astype(np.float32))
    xs = [rnd(rng.standard_normal((n, cfg.D)).astype(np.float32)) for n in ns]
    ms = [rnd(rng.standard_normal((n, dm)).astype(np.float32)) for n in ns]
    if dup:
        for m in ms:
            for k in (1, 4, 7, 10, 13):                 # 5 exact duplicate pairs (fewer than any r below)
                m[2 * k + 1] = m[2 * k]
    szs = [rng.integers(1, sizes_hi + 1, n).astype(np.int32) for n in ns]
    xp, off = synth.pack(xs, cfg.D)
    mp, _ = synth.pack(ms, dm)
    T = int(off[-1])
    reffs = [orc.removal_count(n, r, cfg.n_lead) for n, r in zip(ns, rs)]
    T_out = T - sum(reffs)
    dt = ctx.torch_dtype
    x_d, m_d = _t(torch, xp, dt), _t(torch, mp, dt)
    s_d = torch.from_numpy(np.concatenate(szs)).to("cuda")
    ws = torch.empty(ctx.otas_merge_workspace_bytes(len(ns), T), dtype=torch.uint8, device="cuda")
    x_out = torch.empty((max(T_out, 1), cfg.D), dtype=dt, device="cuda")
    s_out = torch.empty(max(T_out, 1), dtype=torch.int32, device="cuda")
    ntr = max(sum(reffs), 1)
    tsrc = torch.full((ntr,), -1, dtype=torch.int32, device="cuda")
    tdst = torch.full((ntr,), -1, dtype=torch.int32, device="cuda")
    out_off = ctx.otas_token_merge(x_d, m_d, dm, s_d if sizes_hi > 1 else None, off, rs, ws, x_out, s_out, tsrc, tdst)
    torch.cuda.synchronize()
    gx, gs = x_out.to(torch.float32).cpu().numpy().astype(np.float64), s_out.cpu().numpy()
    hs, hd = tsrc.cpu().numpy(), tdst.cpu().numpy()
    st = "bf16" if cfg.dtype == "bf16" else "f32"
    tr = 0
    for q, n in enumerate(ns):
        x2, s2, src, dst, info = orc.token_merge(xs[q], ms[q], szs[q] if sizes_hi > 1 else None, rs[q], cfg.n_lead)
        k = reffs[q]
        assert out_off[q + 1] - out_off[q] == n - k
        if dup:   # cosines of exact duplicates are 1 up to rounding: their mutual order is not unique
            assert sorted(zip(hs[tr:tr + k].tolist(), hd[tr:tr + k].tolist())) == sorted(zip(src.tolist(), dst.tolist()))
            assert {(2 * j, 2 * j + 1) for j in (1, 4, 7, 10, 13)} <= set(zip(hs[tr:tr + k].tolist(), hd[tr:tr + k].tolist()))
        else:
            assert np.array_equal(hs[tr:tr + k], src) and np.array_equal(hd[tr:tr + k], dst), (q, n, rs[q], info)
        tr += k
        assert np.array_equal(gs[out_off[q]:out_off[q + 1]], s2)
        got = gx[out_off[q]:out_off[q + 1]]
        if cfg.dtype == "f32":
            assert hz.rel_err(got, x2) <= 1e-6
        else:
            ref = orc.round_storage(x2, "bf16")
            # fp32 accumulate then one rounding vs float64 then one rounding: at most one bf16 ulp apart
            assert np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-3)) <= 2 ** -7
            assert np.mean(got != ref) < 0.01


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_token_merge_ragged_and_edge_cases(torch_cuda, lib, dtype):
    torch = torch_cuda
    cfg = synth.config("tiny")
    cfg.dtype = dtype
    ctx, _ = hz.make_context(cfg)
    # ragged lengths spanning several tiles and tails; r = 0, r beyond what can be merged, n = 1, 2, 3
    ns = [201, 197, 2, 3, 1, 64, 267, 130, 5]
    rs = [8, 16, 5, 1, 4, 0, 100, 24, 2]
    _merge_case(torch, ctx, cfg, ns, rs, 64, seed=1)
    _merge_case(torch, ctx, cfg, ns, rs, 80, seed=2, sizes_hi=5)
    _merge_case(torch, ctx, cfg, [197] * 3, [16, 8, 50], 64, seed=3, sizes_hi=3, dup=True)   # planted exact ties
    ctx.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_token_merge_queries_longer_than_the_plan_kernels_lds(torch_cuda, lib, dtype):
    """Queries whose unit metric rows do not fit the plan kernel's 160 KB of LDS (more than 554 tokens at metric
    width 64, 293 at 128) keep them in the workspace instead: same decisions (bit-exact against the oracle), up to
    OTAS_MAX_SEQ = 1024 tokens, mixed with short queries in one call."""
    torch = torch_cuda
    cfg = synth.config("tiny")
    cfg.dtype = dtype
    ctx, _ = hz.make_context(cfg)
    _merge_case(torch, ctx, cfg, [555, 40, 1024, 577, 3], [16, 8, 600, 100, 1], 64, seed=11)
    _merge_case(torch, ctx, cfg, [294, 1000, 9], [50, 24, 2], 128, seed=12, sizes_hi=4)
    _merge_case(torch, ctx, cfg, [700], [350], 80, seed=13)
    ctx.close()


@pytest.mark.parametrize("dtype,tol", [("f32", 2e-6), ("bf16", 1e-2)])
def test_layer_norm_linear_attention_steps(torch_cuda, lib, dtype, tol):
    torch = torch_cuda
    cfg = synth.config("tiny")
    cfg.dtype = dtype
    ctx, layers = hz.make_context(cfg)
    dt = ctx.torch_dtype
    rng = np.random.default_rng(7)
    rnd = synth.round_to_bf16 if dtype == "bf16" else (lambda a: a.astype(np.float32))
    T, D, H = 333, cfg.D, cfg.H
    x = rnd((rng.standard_normal((T, D)) * 2 + 0.3).astype(np.float32))
    w = layers[0]
    st = "bf16" if dtype == "bf16" else "f64"
    # LayerNorm
    y = torch.empty((T, D), dtype=dt, device="cuda")
    ctx.otas_layer_norm(_t(torch, x, dt), _t(torch, w["ln1_g"], dt), _t(torch, w["ln1_b"], dt), T, y)
    ref = orc.layer_norm(x.astype(np.float64), w["ln1_g"], w["ln1_b"], cfg.ln_eps)
    assert hz.rel_err(y.to(torch.float32).cpu().numpy(), ref) <= tol
    # Linear with each epilogue, M with a ragged tail
    h = rnd(ref.astype(np.float32))
    for epi, (wn, bn) in enumerate([("w_qkv", "b_qkv"), ("w_fc1", "b_fc1"), ("w_proj", "b_proj")]):
        N = w[wn].shape[0]
        out = torch.empty((T, N), dtype=torch.float32 if epi == 2 else dt, device="cuda")
        res = rng.standard_normal((T, N)).astype(np.float32)
        ctx.otas_linear(_t(torch, h, dt), _t(torch, w[wn], dt), _t(torch, w[bn], dt),
                        _t(torch, res, torch.float32) if epi == 2 else None, T, N, D, epi, out)
        lin = h.astype(np.float64) @ w[wn].astype(np.float64).T + w[bn]
        lin = orc.gelu(lin) if epi == 1 else (lin + res if epi == 2 else lin)
        assert hz.rel_err(out.to(torch.float32).cpu().numpy(), lin) <= tol, wn
    # Attention over a ragged batch, with and without the size bias
    ns = [1, 2, 70, 197, 63]
    off = np.concatenate([[0], np.cumsum(ns)]).astype(np.int32)
    qkv = rnd(rng.standard_normal((int(off[-1]), 3 * D)).astype(np.float32))
    sizes = rng.integers(1, 5, int(off[-1])).astype(np.int32)
    for flags in (0, lib.OTAS_FLAG_SIZE_BIAS):
        o = torch.empty((int(off[-1]), D), dtype=dt, device="cuda")
        ctx.otas_attention(_t(torch, qkv, dt), torch.from_numpy(sizes).to("cuda"), off, flags, o)
        got = o.to(torch.float32).cpu().numpy()
        for q, n in enumerate(ns):
            sl = slice(off[q], off[q + 1])
            ref = orc.attention_heads(qkv[sl].astype(np.float64), H, sizes[sl], bool(flags))
            assert hz.rel_err(got[sl], ref) <= tol, (q, flags)
    ctx.close()


@pytest.mark.parametrize("D,H", [(128, 2), (160, 2), (192, 2), (256, 2), (768, 12)])
def test_attention_bf16_head_widths_and_long_sequences(torch_cuda, lib, D, H):
    """Head widths 64 / 80 / 96 / 128, sequences that span several 256-key chunks and ragged tails."""
    torch = torch_cuda
    cfg = synth.Config("attn", L=1, D=D, H=H, F=2 * D, dtype="bf16", B=1, n0=8, strategies=[(0, 0)], seed=11)
    ctx, _ = hz.make_context(cfg)
    rng = np.random.default_rng(D + H)
    # the longest query picks the kernel's shape for the whole batch: beyond 256 rows (also just beyond: 257 tokens
    # are a 224-pixel image at patch 14), 129 .. 256, up to 128
    for ns in ([1, 33, 197, 256, 257, 300, 700, 129], [257, 267, 320, 300, 161, 160, 31, 289], [197, 256, 130, 7],
               [128, 64, 97, 2]):
        off = np.concatenate([[0], np.cumsum(ns)]).astype(np.int32)
        qkv = synth.round_to_bf16(rng.standard_normal((int(off[-1]), 3 * D)).astype(np.float32))
        sizes = rng.integers(1, 6, int(off[-1])).astype(np.int32)
        for flags in (0, lib.OTAS_FLAG_SIZE_BIAS):
            o = torch.full((int(off[-1]), D), float("nan"), dtype=torch.bfloat16, device="cuda")
            ctx.otas_attention(_t(torch, qkv, torch.bfloat16), torch.from_numpy(sizes).to("cuda"), off, flags, o)
            got = o.to(torch.float32).cpu().numpy()
            assert np.isfinite(got).all()
            for q, n in enumerate(ns):
                sl = slice(off[q], off[q + 1])
                ref = orc.attention_heads(qkv[sl].astype(np.float64), H, sizes[sl], bool(flags))
                assert hz.rel_err(got[sl], ref) <= 1e-2, (q, n, flags)
    ctx.close()


# ------------------------------------------------------------------ whole encoder, bf16 configs
# Near-tie threshold for end-to-end runs: tests/test_bf16_noise_floor.py shows on the CPU that the
# oracle disagrees with a copy of itself fed an input moved by ONE bf16 unit on ~0.5-1 % of the
# merge decisions of a 12-layer run, all within NEAR_TIE of its own choice, with outputs ~1 %
# apart.  End to end the GPU is held to that floor; the 0.1 % bar on decisions is applied where
# both sides see identical inputs (block by block).
from tests.test_bf16_noise_floor import NEAR_TIE


def _bf16_case(cfg, queries):
    ctx, layers = hz.make_context(cfg)
    toks, prm, P, R = synth.batch(cfg, queries)
    x0, off = hz.gpu_prepend(ctx, toks, prm)
    gpu = hz.gpu_forward(ctx, x0, off, R)
    rep = hz.compare_lockstep(cfg, layers, toks, prm, R, gpu)
    for q, qi in enumerate(queries):
        want = orc.length_schedule(cfg.n0, P[q], R[q], cfg.n_lead, cfg.L)[-1]
        assert gpu["x"][q].shape == (want, cfg.D)
        assert int(gpu["sizes"][q].sum()) == cfg.n0 + P[q]
    per = hz.compare_per_layer(ctx, cfg, layers, toks, prm, R)
    ctx.close()
    return rep, per


# Queries per case: enough that 0.1 % of the case's merge decisions is at least one decision
# (186 per vitb_r16 query, 96 per vitb_p10_r8 query), four of every (P, r) group of vitl_ragged and one
# query of each of the eight (P, r) pairs of vith_mixed: (0,0) (0,4) (0,8) (0,12) (10,0) (10,4) (10,8) (10,12).
BF16_CASES = [
    ("vitb_plain", [0, 1]),
    ("vitb_r16", [0, 1, 2, 3, 4, 5]),
    ("vitb_p10_r8", list(range(11))),
    ("vitl_ragged", [0, 1, 2, 3, 32, 33, 34, 35, 64, 65, 66, 67, 96, 97, 98, 99]),
    ("vith_mixed", [6, 3, 7, 4, 5, 0, 2, 12]),
]


@pytest.mark.parametrize("name,queries", BF16_CASES)
def test_bf16_encoder_parity(torch_cuda, lib, name, queries):
    cfg = synth.config(name)
    rep, per = _bf16_case(cfg, queries)
    print(name, "end-to-end lock-step:", rep)
    print(name, "per layer, identical inputs:", per)
    # end to end: values within tolerance under the adopted decisions, sizes identical, and every
    # differing edge a near-tie in the oracle's own similarities
    assert rep["sizes_equal"]
    assert rep["max_err"] <= BF16_TOL
    assert rep["elem_err"] <= BF16_ELEM_TOL
    assert rep["max_deficit"] <= NEAR_TIE
    assert rep["disagreements"] <= BF16_E2E_DECISION_TOL * rep["decisions"]
    # per layer on identical inputs: < 0.1 % of merge decisions differ (no slack: every case that
    # merges has at least 1000 decisions), values within tolerance
    assert per["decisions"] == 0 or per["decisions"] >= 1000
    assert per["sizes_equal"]
    assert per["max_err"] <= BF16_TOL
    assert per["elem_err"] <= BF16_ELEM_TOL
    assert per["disagreements"] <= BF16_DECISION_TOL * per["decisions"]
    print(name, "block-by-block decision disagreement: %d of %d = %.3f %% (bar 0.1 %%)"
          % (per["disagreements"], per["decisions"], 100.0 * per["disagreements"] / max(per["decisions"], 1)))


# ------------------------------------------------------------------ full batches, as bench.py launches them
# Samples: every 4th query of the ViT-B batches (>= 1500 decisions where the strategy merges), four
# queries of every (P, r) group of vitl_ragged, two of each of vith_mixed's eight (P, r) pairs.
FULL_CASES = [
    ("vitb_plain", [0, 63]),
    ("vitb_r16", list(range(0, 64, 4))),
    ("vitb_p10_r8", list(range(0, 64, 4))),
    ("vitl_ragged", [0, 9, 18, 31, 32, 41, 50, 63, 64, 73, 82, 95, 96, 105, 114, 127]),
    ("vith_mixed", [6, 10, 3, 38, 7, 9, 4, 15, 5, 11, 0, 1, 2, 14, 12, 23]),
]


@pytest.mark.parametrize("name,sample", FULL_CASES)
def test_full_batch_sampled_queries(torch_cuda, lib, name, sample):
    """The whole batch of the workload in one launch (the configuration bench.py times); queries are
    independent, so a sample of them is checked against the oracle one by one, in lock-step."""
    cfg = synth.config(name)
    ctx, layers = hz.make_context(cfg)
    toks, prm, P, R = synth.batch(cfg)
    x0, off = hz.gpu_prepend(ctx, toks, prm)
    gpu = hz.gpu_forward(ctx, x0, off, R)
    # shape laws for every query of the batch
    for q in range(cfg.B):
        want = orc.length_schedule(cfg.n0, P[q], R[q], cfg.n_lead, cfg.L)[-1]
        assert gpu["x"][q].shape == (want, cfg.D)
        assert int(gpu["sizes"][q].sum()) == cfg.n0 + P[q] and gpu["sizes"][q].min() >= 1
        assert np.isfinite(gpu["x"][q]).all()
    sub = {k: [gpu[k][q] for q in sample] for k in ("x", "sizes", "trace")}
    rep = hz.compare_lockstep(cfg, layers, [toks[q] for q in sample], [prm[q] for q in sample],
                              [R[q] for q in sample], sub)
    print(name, "full batch, sampled", sample, rep)
    assert rep["sizes_equal"]
    assert rep["max_err"] <= BF16_TOL
    assert rep["elem_err"] <= BF16_ELEM_TOL
    assert rep["max_deficit"] <= NEAR_TIE
    assert rep["decisions"] == 0 or rep["decisions"] >= 1500
    assert rep["disagreements"] <= BF16_E2E_DECISION_TOL * rep["decisions"]
    ctx.close()


def test_bf16_path_against_the_unrounded_oracle(torch_cuda, lib):
    """The absolute error of the bf16 path: the plain ViT-B encoder (no merging, so no decisions to
    adopt) against the oracle in float64 WITHOUT storage rounding.  This is the error of computing in
    bf16 at all, not a parity bar of the kernels (those are held to the bf16-storage oracle above);
    measured 2.3e-3 for the GPU and for the bf16-storage oracle alike."""
    cfg = synth.config("vitb_plain")
    ctx, layers = hz.make_context(cfg)
    qs = [0, 17, 40, 63]
    toks, prm, P, R = synth.batch(cfg, qs)
    x0, off = hz.gpu_prepend(ctx, toks, prm)
    gpu = hz.gpu_forward(ctx, x0, off, R)
    exact = hz.oracle_forward(cfg, layers, toks, prm, R, storage="f64")
    stored = hz.oracle_forward(cfg, layers, toks, prm, R, storage="bf16")
    e_gpu = max(hz.rel_err(gpu["x"][i], exact[i]["x"]) for i in range(len(qs)))
    e_orc = max(hz.rel_err(stored[i]["x"], exact[i]["x"]) for i in range(len(qs)))
    e_par = max(hz.rel_err(gpu["x"][i], stored[i]["x"]) for i in range(len(qs)))
    print("vitb_plain bf16 vs float64 without rounding: GPU %.3e, bf16-storage oracle %.3e; GPU vs bf16-storage oracle %.3e"
          % (e_gpu, e_orc, e_par))
    assert e_par <= BF16_TOL
    assert e_gpu <= 1e-2 and e_gpu <= 2.0 * e_orc + 1e-3    # the kernels add nothing beyond the storage rounding
    ctx.close()


def test_edge_cases_through_the_abi(torch_cuda, lib):
    """Degenerate inputs: one query of one token, sequences at the floor, r beyond what can merge,
    no protected token, a single-query batch."""
    torch = torch_cuda
    for n_lead in (1, 0):
        cfg = synth.Config("edge", L=3, D=192, H=3, F=384, dtype="f32", B=5, n0=9,
                           strategies=[(0, 0), (0, 50), (2, 1), (0, 3), (1, 50)], seed=21, n_lead=n_lead)
        ctx, layers = hz.make_context(cfg)
        rng = np.random.default_rng(5)
        ns = [1, 9, 2, 3, 40]
        toks = [rng.standard_normal((n, cfg.D)).astype(np.float32) for n in ns]
        prm = [(0.02 * rng.standard_normal((p, cfg.D))).astype(np.float32) for p, _ in cfg.strategies]
        R = [r for _, r in cfg.strategies]
        x0, off = hz.gpu_prepend(ctx, toks, prm)
        gpu = hz.gpu_forward(ctx, x0, off, R)
        for q in range(cfg.B):
            xq, _ = orc.prompt_prepend(toks[q], prm[q], n_lead)
            ref = orc.encoder_forward_query(xq, layers, R[q], H=cfg.H, ln_eps=cfg.ln_eps, n_lead=n_lead)
            assert gpu["x"][q].shape == ref["x"].shape, (n_lead, q)
            assert np.array_equal(gpu["sizes"][q], ref["sizes"]), (n_lead, q)
            for l in range(cfg.L):
                assert np.array_equal(gpu["trace"][q][l][0], ref["trace"][l][0]), (n_lead, q, l)
                assert np.array_equal(gpu["trace"][q][l][1], ref["trace"][l][1]), (n_lead, q, l)
            assert hz.rel_err(gpu["x"][q], ref["x"]) <= F32_TOL, (n_lead, q)
        ctx.close()


def test_argument_errors_on_the_gpu_box(torch_cuda, lib):
    torch = torch_cuda
    cfg = synth.config("tiny")
    ctx, _ = hz.make_context(cfg)
    x0 = torch.zeros((10, cfg.D), dtype=torch.float32, device="cuda")
    ws = torch.empty(ctx.otas_workspace_bytes(1, 10), dtype=torch.uint8, device="cuda")
    xo = torch.empty((10, cfg.D), dtype=torch.float32, device="cuda")
    so = torch.empty(10, dtype=torch.int32, device="cuda")
    with pytest.raises(lib.OtasError) as e:                         # workspace too small
        ctx.otas_encoder_forward(x0, [0, 10], [1], 0, ws[:1024], xo, so)
    assert e.value.status == 3
    with pytest.raises(lib.OtasError) as e:                         # offsets not starting at 0
        ctx.otas_encoder_forward(x0, [1, 10], [1], 0, ws, xo, so)
    assert e.value.status == 1
    with pytest.raises(lib.OtasError) as e:                         # negative r
        ctx.otas_encoder_forward(x0, [0, 10], [-1], 0, ws, xo, so)
    assert e.value.status == 1
    with pytest.raises(lib.OtasError) as e:                         # unknown flag
        ctx.otas_encoder_forward(x0, [0, 10], [1], 64, ws, xo, so)
    assert e.value.status == 1
    with pytest.raises(lib.OtasError) as e:                         # trace flag without buffers
        ctx.otas_encoder_forward(x0, [0, 10], [1], lib.OTAS_FLAG_TRACE, ws, xo, so)
    assert e.value.status == 1
    with pytest.raises(lib.OtasError) as e:                         # sequence longer than the kernels take
        big = torch.zeros((1100, cfg.D), dtype=torch.float32, device="cuda")
        ctx.otas_encoder_forward(big, [0, 1100], [1], 0, torch.empty(ctx.otas_workspace_bytes(1, 1100), dtype=torch.uint8, device="cuda"),
                                 torch.empty((1100, cfg.D), dtype=torch.float32, device="cuda"), torch.empty(1100, dtype=torch.int32, device="cuda"))
    assert e.value.status == 5
    # a failed call enqueued nothing: the context still works
    off = ctx.otas_encoder_forward(x0, [0, 10], [1], 0, ws, xo, so)
    torch.cuda.synchronize()
    assert off.tolist() == [0, 8]
    ctx.close()


def _same_trace(a, b):
    return len(a) == len(b) and all(np.array_equal(x[0], y[0]) and np.array_equal(x[1], y[1]) for x, y in zip(a, b))


def test_query_independence_of_batch_composition(torch_cuda, lib):
    """A query's result must not depend on what else is in the ragged batch.  The fp32 path computes
    every row the same way whatever the batch, so there the results are identical; the bf16 GEMMs
    pick tile shapes and the split-K factor from the batch's row count, which changes the order of
    the fp32 accumulation, so there the results agree to the bf16 tolerance (compared without
    merging, where no near-tie decision can amplify the rounding difference)."""
    cfg = synth.config("tiny")
    cfg.B = 4
    cfg.strategies = [(4, 8), (0, 16), (0, 0), (4, 0)]
    ctx, layers = hz.make_context(cfg)
    toks, prm, P, R = synth.batch(cfg, [0, 1, 2, 3])
    x0, off = hz.gpu_prepend(ctx, toks, prm)
    together = hz.gpu_forward(ctx, x0, off, R)
    for q in range(4):
        x1, off1 = hz.gpu_prepend(ctx, toks[q:q + 1], prm[q:q + 1])
        alone = hz.gpu_forward(ctx, x1, off1, R[q:q + 1])
        assert np.array_equal(alone["sizes"][0], together["sizes"][q])
        assert _same_trace(alone["trace"][0], together["trace"][q])
        assert hz.rel_err(alone["x"][0], together["x"][q]) <= 1e-6
    ctx.close()

    cfg = synth.config("vitb_p10_r8")
    cfg.strategies = [(10, 0), (0, 0)] * 2 + cfg.strategies[4:]
    ctx, layers = hz.make_context(cfg)
    toks, prm, P, R = synth.batch(cfg, [0, 1, 2, 3])
    x0, off = hz.gpu_prepend(ctx, toks, prm)
    together = hz.gpu_forward(ctx, x0, off, R)
    for q in range(4):
        x1, off1 = hz.gpu_prepend(ctx, toks[q:q + 1], prm[q:q + 1])
        alone = hz.gpu_forward(ctx, x1, off1, R[q:q + 1])
        assert np.array_equal(alone["sizes"][0], together["sizes"][q])
        assert hz.rel_err(alone["x"][0], together["x"][q]) <= BF16_TOL
    ctx.close()


def test_lanes_do_not_change_results(torch_cuda, lib):
    """Cutting the batch into lanes that run side by side changes nothing in the fp32 model (bit for
    bit: x, sizes, trace) and stays within the bf16 tolerance in the bf16 model without merging."""
    cfg = synth.config("tiny")
    cfg.B = 7
    cfg.strategies = [(4, 8), (0, 16), (0, 0), (4, 0), (2, 3), (0, 5), (1, 1)]
    ctx, layers = hz.make_context(cfg)
    toks, prm, P, R = synth.batch(cfg, list(range(7)))
    x0, off = hz.gpu_prepend(ctx, toks, prm)
    ctx.otas_set_lanes(1)
    ref = hz.gpu_forward(ctx, x0, off, R)
    for lanes in (2, 3, 7, 8):
        ctx.otas_set_lanes(lanes)
        got = hz.gpu_forward(ctx, x0, off, R)
        for q in range(7):
            assert np.array_equal(got["x"][q], ref["x"][q]), (lanes, q)
            assert np.array_equal(got["sizes"][q], ref["sizes"][q])
            assert _same_trace(got["trace"][q], ref["trace"][q])
    with pytest.raises(lib.OtasError):
        ctx.otas_set_lanes(9)
    ctx.close()

    cfg = synth.config("vitb_p10_r8")
    cfg.B = 6
    cfg.strategies = [(10, 0), (0, 0)] * 3
    ctx, layers = hz.make_context(cfg)
    toks, prm, P, R = synth.batch(cfg, list(range(6)))
    x0, off = hz.gpu_prepend(ctx, toks, prm)
    ctx.otas_set_lanes(1)
    ref = hz.gpu_forward(ctx, x0, off, R)
    ctx.otas_set_lanes(3)
    got = hz.gpu_forward(ctx, x0, off, R)
    for q in range(6):
        assert hz.rel_err(got["x"][q], ref["x"][q]) <= BF16_TOL
    ctx.close()


def test_lanes_bit_identical_full_batch_bf16(torch_cuda, lib):
    """Full ViT-B batch without merging.  A lane's kernels are chosen from the lane's row counts, so the
    rows of every lane of a G-lane run -- different tile shapes per lane, kernels of different lanes
    sharing CUs -- must equal, bit for bit, a single-lane call on that lane's queries alone; and where no
    lane splits a product over K (1 and 2 lanes here) the whole result equals the single-lane one.
    Guards the kernels' LDS stage reuse against co-resident workgroups."""
    import torch
    cfg = synth.config("vitb_plain")
    ctx, layers = hz.make_context(cfg)
    toks, prm, P, R = synth.batch(cfg)
    x0, off = hz.gpu_prepend(ctx, toks, prm)
    off = np.asarray(off, dtype=np.int64)
    T0, B = int(off[-1]), cfg.B
    ws = torch.empty(ctx.otas_workspace_bytes(B, T0), dtype=torch.uint8, device="cuda")

    def run(q0, q1, lanes):
        ctx.otas_set_lanes(lanes)
        r0, r1 = int(off[q0]), int(off[q1])
        x_out = torch.zeros((r1 - r0, cfg.D), dtype=torch.float32, device="cuda")
        sz = torch.zeros(r1 - r0, dtype=torch.int32, device="cuda")
        ctx.otas_encoder_forward(x0[r0:r1].contiguous(), (off[q0:q1 + 1] - r0).astype(np.int32), R[q0:q1], 0, ws, x_out, sz)
        torch.cuda.synchronize()
        return x_out

    def lane_ranges(G):   # the rule of otas_set_lanes: lane g ends where the token count reaches T0 (g + 1) / G
        cuts, q = [0], 0
        for g in range(G - 1):
            goal = T0 * (g + 1) // G
            q += 1
            while q < B - (G - 1 - g) and off[q] < goal:
                q += 1
            cuts.append(q)
        return list(zip(cuts, cuts[1:] + [B]))

    whole = run(0, B, 1)
    for G in (3, 2, 3):
        got = run(0, B, G)
        ranges = lane_ranges(G)
        for q0, q1 in ranges:
            assert torch.equal(got[int(off[q0]):int(off[q1])], run(q0, q1, 1)), (G, q0, q1)
        if all(ctx.otas_splitk_factor(int(off[q1] - off[q0]), cfg.D, cfg.F, ctx.otas_splitk_room(int(off[q1] - off[q0]), int(off[q1] - off[q0]))) == 1 for q0, q1 in ranges):
            assert torch.equal(got, whole), G
    assert ctx.otas_splitk_factor(T0, cfg.D, cfg.F, 2) == 1 and ctx.otas_splitk_factor(T0 // 2, cfg.D, cfg.F, 2) == 1
    ctx.close()


@pytest.mark.parametrize("M,N,K,epi", [
    (12608, 2304, 768, 0), (10560, 2304, 768, 0), (8512, 2304, 768, 0),      # 256-, 192-, 320-row tiles
    (12608 + 37, 3072, 768, 1), (10560 - 3, 768, 3072, 2), (4416 + 5, 768, 768, 2),
    (1344, 768, 3072, 2), (67, 2304, 768, 0), (12608, 768, 3072, 2)])
def test_linear_bf16_every_kernel_ragged_rows(torch_cuda, lib, M, N, K, epi):
    """otas_linear at the encoder's own shapes, chosen so that every MFMA kernel and tile height the
    dispatch knows is exercised, with row counts that leave ragged last tiles.  The WHOLE output is
    compared with a float64 product."""
    torch = torch_cuda
    cfg = synth.config("vitb_plain")
    cfg.L = 1
    ctx, layers = hz.make_context(cfg)
    rng = np.random.default_rng(M + N + K + epi)
    x = synth.round_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
    w = synth.round_to_bf16((rng.standard_normal((N, K)) * 0.03).astype(np.float32))
    b = synth.round_to_bf16((rng.standard_normal(N) * 0.1).astype(np.float32))
    res = rng.standard_normal((M, N)).astype(np.float32)
    dt = torch.bfloat16
    out = torch.full((M, N), float("nan"), dtype=torch.float32 if epi == 2 else dt, device="cuda")
    ctx.otas_linear(_t(torch, x, dt), _t(torch, w, dt), _t(torch, b, dt),
                    _t(torch, res, torch.float32) if epi == 2 else None, M, N, K, epi, out)
    got = out.to(torch.float32).cpu().numpy()
    assert np.isfinite(got).all()
    lin = x.astype(np.float64) @ w.astype(np.float64).T + b
    lin = orc.gelu(lin) if epi == 1 else (lin + res if epi == 2 else lin)
    if epi == 2:      # float output: only the fp32 accumulation order separates the two
        assert hz.rel_err(got, lin) <= 1e-5 and hz.elem_err(got, lin) <= 1e-4
    else:             # bf16 output: one rounding of the float64 value, up to the last place
        assert hz.rel_err(got, lin) <= 2.0 ** -8 and hz.elem_err(got, lin) <= 2.0 ** -7
    ctx.close()


def test_gelu_epilogue_over_every_bf16_input_in_range(torch_cuda, lib):
    """The GELU of the MFMA kernels' epilogue (a polynomial for log2 Phi(-|x|) and one exp2, not erf) on EVERY
    bf16 value in [-9, 9]: an identity weight and a zero bias make the pre-activation the input itself.  Against
    the exact erf form in float64: the absolute error before the result is rounded to bf16 is within 4e-7, so
    the rounded result is within half a bf16 unit + 4e-7 of the exact value everywhere, and equals the correctly
    rounded value for all but a small share of the inputs."""
    torch = torch_cuda
    cfg = synth.config("vitb_plain")
    cfg.L = 1
    ctx, _ = hz.make_context(cfg)
    bits = np.arange(0, 1 << 16, dtype=np.uint32)
    vals = (bits << 16).view(np.float32)
    vals = vals[np.isfinite(vals) & (np.abs(vals) <= 9.0)]
    K = 256
    M = -(-vals.size // K)
    x = np.zeros(M * K, dtype=np.float32)
    x[:vals.size] = vals
    x = x.reshape(M, K)
    w = np.eye(K, dtype=np.float32)
    out = torch.full((M, K), float("nan"), dtype=torch.bfloat16, device="cuda")
    ctx.otas_linear(_t(torch, x, torch.bfloat16), _t(torch, w, torch.bfloat16),
                    torch.zeros(K, dtype=torch.bfloat16, device="cuda"), None, M, K, K, 1, out)
    got = out.to(torch.float32).cpu().numpy().astype(np.float64)
    ref = orc.gelu(x.astype(np.float64))
    half_unit = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 1e-30))) - 8)     # half a bf16 unit at the exact value
    assert np.all(np.abs(got - ref) <= half_unit + 4e-7)
    exact_rounded = synth.round_to_bf16(ref.astype(np.float32)).astype(np.float64)
    big = np.abs(ref) > 1e-4                                                       # below that 4e-7 is whole bf16 units
    share = float(np.mean(got[big] != exact_rounded[big]))
    print("share of inputs whose GELU is not the correctly rounded bf16 value: %.4f %%" % (100 * share))
    assert share <= 1e-3          # measured 2.6e-4
    assert np.all(got[x >= 8.0] == x[x >= 8.0].astype(np.float64)) and np.all(np.abs(got[x <= -8.0]) <= 1e-6)
    ctx.close()


@pytest.mark.parametrize("kernel", range(1, 8))
def test_linear_every_named_kernel_whole_output(torch_cuda, lib, kernel):
    """Every GEMM kernel of the library forced by name (otas_linear_kernel) on shapes with ragged row
    and column tiles, all three epilogues, the whole output against a float64 product; a K that a
    kernel does not take is refused, not mangled."""
    torch = torch_cuda
    cfg = synth.config("vitb_plain")
    cfg.L = 1
    ctx, layers = hz.make_context(cfg)
    dt = torch.bfloat16
    for M, N, K, epi in [(1345, 776, 768, 2), (701, 2304, 256, 0), (523, 1000, 768, 1), (389, 768, 3072, 2), (33, 8, 128, 0)]:
        rng = np.random.default_rng(M + N + K + epi + kernel)
        x = synth.round_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
        w = synth.round_to_bf16((rng.standard_normal((N, K)) * 0.03).astype(np.float32))
        b = synth.round_to_bf16((rng.standard_normal(N) * 0.1).astype(np.float32))
        res = rng.standard_normal((M, N)).astype(np.float32)
        out = torch.full((M, N), float("nan"), dtype=torch.float32 if epi == 2 else dt, device="cuda")
        ctx.otas_linear_kernel(kernel, _t(torch, x, dt), _t(torch, w, dt), _t(torch, b, dt),
                               _t(torch, res, torch.float32) if epi == 2 else None, M, N, K, epi, out)
        got = out.to(torch.float32).cpu().numpy()
        lin = x.astype(np.float64) @ w.astype(np.float64).T + b
        lin = orc.gelu(lin) if epi == 1 else (lin + res if epi == 2 else lin)
        assert np.isfinite(got).all(), (kernel, M, N, K, epi)
        if epi == 2:
            assert hz.rel_err(got, lin) <= 1e-5 and hz.elem_err(got, lin) <= 1e-4, (kernel, M, N, K, epi)
        else:
            assert hz.rel_err(got, lin) <= 2.0 ** -8 and hz.elem_err(got, lin) <= 2.0 ** -7, (kernel, M, N, K, epi)
    if kernel >= 2:     # MFMA kernels: K = 96 suits only the K-step-32 kernels, K = 40 none of them
        x = torch.zeros((64, 96), dtype=dt, device="cuda")
        w = torch.zeros((64, 96), dtype=dt, device="cuda")
        b = torch.zeros(64, dtype=dt, device="cuda")
        y = torch.zeros((64, 64), dtype=dt, device="cuda")
        if kernel in (2, 7):
            ctx.otas_linear_kernel(kernel, x, w, b, None, 64, 64, 96, 0, y)
        else:
            with pytest.raises(lib.OtasError) as e:
                ctx.otas_linear_kernel(kernel, x, w, b, None, 64, 64, 96, 0, y)
            assert e.value.status == 5
        with pytest.raises(lib.OtasError):
            ctx.otas_linear_kernel(kernel, x[:, :40].contiguous(), w[:, :40].contiguous(), b, None, 64, 64, 40, 0, y)
    torch.cuda.synchronize()
    ctx.close()


def test_longest_sequences_f32(torch_cuda, lib):
    """Long merging queries next to a short one, fp32, r larger than half the tokens: 554 tokens (the longest
    whose unit metric vectors fit the plan kernel's LDS at d_h = 64), 577 (a 384-pixel image at patch 16: the
    metric rows then live in the workspace) and 1024 (OTAS_MAX_SEQ).  Decisions checked against the oracle in
    lock-step (bit-exact unless the oracle itself sees an exact tie); 1025 tokens are refused."""
    torch = torch_cuda
    cfg = synth.config("tiny")
    cfg.n0 = 1020
    cfg.strategies = [(4, 600), (0, 3)]
    ctx, layers = hz.make_context(cfg)
    long_tok = synth.query_tokens(cfg, 0)
    prm = [synth.query_prompts(cfg, 0), synth.query_prompts(cfg, 1)]
    R = [600, 3]
    for n_long, want in ((554, [0, 140, 144]), (577, [0, 145, 149]), (1024, [0, 257, 261])):
        toks = [long_tok[:n_long - 4], synth.query_tokens(cfg, 1)[:9]]
        x0, off = hz.gpu_prepend(ctx, toks, prm)
        assert off.tolist() == [0, n_long, n_long + 9]
        gpu = hz.gpu_forward(ctx, x0, off, R)
        rep = hz.compare_lockstep(cfg, layers, toks, prm, R, gpu)
        print(f"n = {n_long}:", rep)
        assert rep["sizes_equal"] and rep["max_err"] <= F32_TOL
        assert rep["disagreements"] == 0 or rep["max_deficit"] <= 1e-6
        assert gpu["offsets"].tolist() == want   # n -> ceil(n / 2) + ... twice; 9 -> 6 -> 4 (r clamps to 2)
    # no merging: the full 1024 tokens
    x2, off2 = hz.gpu_prepend(ctx, [long_tok], [prm[0]])
    assert off2.tolist() == [0, 1024]
    g2 = hz.gpu_forward(ctx, x2, off2, [0])
    cfg.strategies = [(4, 0)]
    ref = hz.oracle_forward(cfg, layers, [long_tok], [prm[0]], [0])
    assert hz.rel_err(g2["x"][0], ref[0]["x"]) <= F32_TOL
    ctx.close()


def test_long_ragged_sequences_bf16_plan_split_over_two_launches(torch_cuda, lib):
    """bf16, head width 64, H = 4: the encoder runs the merge plan's selection beside attention and writes its lists
    beside the output projection (256 threads there: a 554-token query gives every thread three positions of the
    scans; 554 is the longest query this path takes).  Ragged lengths 554 / 300 / 130 / 9, r up to 100, one query that
    merges nothing.  Lock-step against the oracle: sizes identical, every differing edge a near-tie."""
    torch = torch_cuda
    cfg = synth.config("tiny")
    cfg.D, cfg.H, cfg.F, cfg.dtype, cfg.n0, cfg.L, cfg.B = 256, 4, 512, "bf16", 554, 3, 5
    cfg.strategies = [(0, 100), (4, 37), (0, 16), (0, 3), (2, 0)]
    ctx, layers = hz.make_context(cfg)
    lens = [554, 296, 130, 9, 75]
    toks = [synth.query_tokens(cfg, q)[:n] for q, n in enumerate(lens)]
    prm = [synth.query_prompts(cfg, q) for q in range(cfg.B)]
    R = [r for _, r in cfg.strategies]
    x0, off = hz.gpu_prepend(ctx, toks, prm)
    assert np.diff(off).tolist() == [554, 300, 130, 9, 77]
    gpu = hz.gpu_forward(ctx, x0, off, R)
    rep = hz.compare_lockstep(cfg, layers, toks, prm, R, gpu)
    print(rep)
    assert rep["sizes_equal"] and rep["max_err"] <= BF16_TOL and rep["max_deficit"] <= NEAR_TIE
    assert np.diff(gpu["offsets"]).tolist() == [254, 189, 82, 3, 77]   # 9 -> 6 -> 4 -> 3: r clamps to half the unprotected tokens
    ctx.close()


def test_splitk_factor_and_room_are_consistent(torch_cuda, lib):
    """The split factor of the MLP's second linear is one of 1, 2, 3, 4, 6, 8, never above the room the caller
    names, 1 for f32 models and for full ViT-B batches; the room is two partial rows per token row, up to eight for
    batches of at most 1024 rows, never below 1 or above 8."""
    cfg = synth.config("vitb_plain")
    cfg.L = 1
    ctx, _ = hz.make_context(cfg)
    for M in (1, 64, 197, 704, 1344, 2368, 3392, 4416, 5440, 8512, 12608, 67072):
        for room in (1, 2, 3, 5, 8):
            S = ctx.otas_splitk_factor(M, cfg.D, cfg.F, room)
            assert S in (1, 2, 3, 4, 6, 8) and S <= room, (M, room, S)
    assert ctx.otas_splitk_factor(12608, cfg.D, cfg.F, 8) == 1
    assert ctx.otas_splitk_factor(197, cfg.D, cfg.F, 8) > 1
    assert ctx.otas_splitk_factor(197, cfg.D, cfg.D, 8) == 1          # K = 768: never split
    assert [ctx.otas_splitk_room(T0, T0) for T0 in (197, 1024, 1025, 2048, 2049, 4096, 12608)] == [8, 8, 6, 4, 3, 2, 2]
    assert ctx.otas_splitk_room(12608, 704) == 8 and ctx.otas_splitk_room(12608, 5440) == 4
    assert ctx.otas_splitk_room(12608, 10 ** 9) == 1
    ctx.close()
    cfg32 = synth.config("tiny")
    ctx32, _ = hz.make_context(cfg32)
    assert ctx32.otas_splitk_factor(197, cfg32.D, 4096, 8) == 1
    ctx32.close()


def test_per_launch_timing_api(torch_cuda, lib):
    """otas_timing_*: one record per launch in launch order, kinds named, the event-pair overhead is
    calibrated and non-negative, records stop when timing is off, and timing changes no result."""
    torch = torch_cuda
    cfg = synth.config("tiny")
    ctx, layers = hz.make_context(cfg)
    toks, prm, P, R = synth.batch(cfg)
    x0, off = hz.gpu_prepend(ctx, toks, prm)
    ref = hz.gpu_forward(ctx, x0, off, R, trace=False)
    ctx.otas_timing_enable(True)
    assert 0.0 <= ctx.otas_timing_overhead_ms() < 0.1
    got = hz.gpu_forward(ctx, x0, off, R, trace=False)
    recs = ctx.otas_timing_read_launches()
    kinds = [k for k, _ in recs]
    per_layer = ["layer_norm", "gemm_qkv", "merge_plan", "attention", "gemm_proj", "merge_apply", "gemm_fc1", "gemm_fc2"]
    assert kinds == per_layer * cfg.L, kinds
    assert all(ms > 0 for _, ms in recs)
    assert set(kinds) <= set(ctx.otas_timing_kind_names())
    totals = ctx.otas_timing_read()
    assert totals["gemm_qkv"][1] == cfg.L and totals["merge_apply"][1] == cfg.L
    ctx.otas_timing_enable(False)
    hz.gpu_forward(ctx, x0, off, R, trace=False)
    assert ctx.otas_timing_read_launches() == []
    for q in range(cfg.B):
        assert np.array_equal(got["x"][q], ref["x"][q]) and np.array_equal(got["sizes"][q], ref["sizes"][q])
    ctx.close()


@pytest.mark.parametrize("mode", ["replace", "grow"])
def test_per_layer_prompting_f32(torch_cuda, lib, mode):
    """otas_encoder_forward_deep in fp32 against the oracle: a ragged batch in which queries carry
    different prompt counts (one none at all), four layers so that the replaced / inserted rows pass
    through several prompting steps."""
    cfg = synth.config("tiny")
    cfg.L = 4
    cfg.B = 4
    cfg.strategies = [(4, 0), (0, 0), (7, 0), (1, 0)]
    cfg.deep = mode
    ctx, layers = hz.make_context(cfg)
    qs = [0, 1, 2, 3]
    gpu = hz.gpu_forward_deep(ctx, cfg, qs, mode)
    ref = hz.oracle_forward_deep(cfg, layers, qs, mode)
    for i, q in enumerate(qs):
        P = cfg.strategies[q][0]
        want = orc.deep_length_schedule(cfg.n0, P, cfg.L, mode)[-1]
        assert gpu["x"][i].shape == ref[i]["x"].shape == (want, cfg.D)
        assert np.all(gpu["sizes"][i] == 1)
        assert hz.rel_err(gpu["x"][i], ref[i]["x"]) <= F32_TOL, (mode, q)
    ctx.close()


@pytest.mark.parametrize("name", ["vitb_deep10_replace", "vitb_deep2_grow"])
def test_per_layer_prompting_bf16_full_batch(torch_cuda, lib, name):
    """The ViT-B per-layer prompting workloads at full batch (the launch configuration bench.py times),
    sampled queries against the oracle."""
    cfg = synth.config(name)
    ctx, layers = hz.make_context(cfg)
    gpu = hz.gpu_forward_deep(ctx, cfg, list(range(cfg.B)), cfg.deep)
    sample = [0, 29, 63]
    ref = hz.oracle_forward_deep(cfg, layers, sample, cfg.deep)
    for i, q in enumerate(sample):
        assert gpu["x"][q].shape == ref[i]["x"].shape
        err = hz.rel_err(gpu["x"][q], ref[i]["x"])
        print(name, "query", q, "rel err", err)
        assert err <= BF16_TOL
    ctx.close()


@pytest.mark.parametrize("name,queries", [("vitl_ragged", [0, 40, 70, 100, 33, 99, 71]),
                                          ("vith_mixed", [12, 4, 2, 7, 23, 15])])
def test_size_bias_on_the_ragged_bf16_workloads(torch_cuda, lib, name, queries):
    """OTAS_FLAG_SIZE_BIAS on the selective batches of ViT-L and ViT-H (queries that merge most, next to
    one that only prompts): block by block on identical inputs the decisions must agree to 0.1 %, end
    to end in lock-step every differing edge must be a near-tie; and the flag must matter."""
    cfg = synth.config(name)
    ctx, layers = hz.make_context(cfg)
    toks, prm, P, R = synth.batch(cfg, queries)
    x0, off = hz.gpu_prepend(ctx, toks, prm)
    gpu = hz.gpu_forward(ctx, x0, off, R, flags=lib.OTAS_FLAG_SIZE_BIAS)
    plain = hz.gpu_forward(ctx, x0, off, R)
    rep = hz.compare_lockstep(cfg, layers, toks, prm, R, gpu, size_bias=True)
    per = hz.compare_per_layer(ctx, cfg, layers, toks, prm, R, size_bias=True)
    print(name, "size bias end to end:", rep)
    print(name, "size bias per layer:", per)
    assert rep["sizes_equal"] and rep["max_err"] <= BF16_TOL and rep["elem_err"] <= BF16_ELEM_TOL
    assert rep["max_deficit"] <= NEAR_TIE
    assert rep["decisions"] >= 1000 and rep["disagreements"] <= BF16_E2E_DECISION_TOL * rep["decisions"]
    assert per["sizes_equal"] and per["max_err"] <= BF16_TOL
    assert per["decisions"] >= 1000 and per["disagreements"] <= BF16_DECISION_TOL * per["decisions"]
    merging = [i for i, r in enumerate(R) if r > 0]
    assert any(hz.rel_err(gpu["x"][i], plain["x"][i]) > 1e-3 for i in merging)
    ctx.close()


@pytest.mark.parametrize("shape,mode", [("vitl_ragged", "replace"), ("vitl_ragged", "grow"),
                                        ("vith_mixed", "replace"), ("vith_mixed", "grow")])
def test_per_layer_prompting_on_the_large_models_ragged_prompts(torch_cuda, lib, shape, mode):
    """Per-layer prompting at the ViT-L and ViT-H shapes with a different prompt count per query
    (0, 2, 5, 10 rows; sequences grow to 197 + 24 * 10 and 257 + 32 * 5 rows) in one launch."""
    base = synth.config(shape)
    Ps = [0, 2, 10, 5] if shape == "vitl_ragged" else [5, 0, 2, 3]
    cfg = synth.Config(shape + "_deep_" + mode, base.L, base.D, base.H, base.F, "bf16", len(Ps), base.n0,
                       [(p, 0) for p in Ps], seed=base.seed + 40, deep=mode)
    ctx, layers = hz.make_context(cfg)
    qs = list(range(cfg.B))
    gpu = hz.gpu_forward_deep(ctx, cfg, qs, mode)
    ref = hz.oracle_forward_deep(cfg, layers, qs, mode)
    for q in qs:
        want = orc.deep_length_schedule(cfg.n0, Ps[q], cfg.L, mode)[-1]
        assert gpu["x"][q].shape == ref[q]["x"].shape == (want, cfg.D)
        assert gpu["sizes"][q].tolist() == [1] * want
        err, eerr = hz.rel_err(gpu["x"][q], ref[q]["x"]), hz.elem_err(gpu["x"][q], ref[q]["x"])
        print(cfg.name, "query", q, "P", Ps[q], "rel err %.2e elem err %.2e" % (err, eerr))
        assert err <= BF16_TOL and eerr <= BF16_ELEM_TOL
    ctx.close()


def test_per_layer_prompting_argument_errors(torch_cuda, lib):
    torch = torch_cuda
    cfg = synth.config("tiny")
    ctx, layers = hz.make_context(cfg)
    x0 = torch.zeros((10, cfg.D), dtype=torch.float32, device="cuda")
    pr = torch.zeros((cfg.L, 3, cfg.D), dtype=torch.float32, device="cuda")
    ws = torch.empty(ctx.otas_workspace_bytes(1, 64), dtype=torch.uint8, device="cuda")
    xo = torch.empty((64, cfg.D), dtype=torch.float32, device="cuda")
    so = torch.empty(64, dtype=torch.int32, device="cuda")
    for bad_mode in (0, 3):
        with pytest.raises(lib.OtasError) as e:
            ctx.otas_encoder_forward_deep(x0, [0, 10], bad_mode, pr, [0, 3], ws, xo, so)
        assert e.value.status == 1
    with pytest.raises(lib.OtasError) as e:      # more prompt rows than the query holds
        ctx.otas_encoder_forward_deep(x0, [0, 3], lib.OTAS_PROMPT_REPLACE, pr, [0, 3], ws, xo, so)
    assert e.value.status == 1
    with pytest.raises(lib.OtasError) as e:      # prompts missing
        ctx.otas_encoder_forward_deep(x0, [0, 10], lib.OTAS_PROMPT_GROW, None, [0, 3], ws, xo, so)
    assert e.value.status == 1
    with pytest.raises(lib.OtasError) as e:      # workspace too small for the grown sequence
        ctx.otas_encoder_forward_deep(x0, [0, 10], lib.OTAS_PROMPT_GROW, pr, [0, 3], ws[:4096], xo, so)
    assert e.value.status == 3
    off = ctx.otas_encoder_forward_deep(x0, [0, 10], lib.OTAS_PROMPT_GROW, pr, [0, 3], ws, xo, so)
    torch.cuda.synchronize()
    assert off.tolist() == [0, 10 + 3 * (cfg.L - 1)]
    ctx.close()


@pytest.mark.parametrize("dtype,tol", [("f32", 2e-6), ("bf16", 1e-2)])
def test_model_ends_patch_embed_and_task_heads(torch_cuda, lib, dtype, tol):
    """Model ends against the oracle: patch embedding of 3 x 64 x 48 images (patch 16: a 4 x 3 grid, so a
    wrong patch order shows) with class token and position embedding, and two task heads of different
    widths reading LayerNorm_final of each query's first row from a ragged float tensor."""
    torch = torch_cuda
    cfg = synth.config("tiny")
    cfg.dtype = dtype
    cfg.B = 3
    ctx, layers = hz.make_context(cfg)
    dt = ctx.torch_dtype
    C, Hi, Wi, p = 3, 64, 48, 16
    N = (Hi // p) * (Wi // p)
    classes = [10, 37]
    ends = synth.ends_weights(cfg, C, p, N, classes)
    imgs = np.stack([synth.query_image(cfg, q, C, Hi, Wi) for q in range(cfg.B)])
    st = "bf16" if dtype == "bf16" else "f64"
    ws = torch.empty(ctx.otas_patch_embed_workspace_bytes(cfg.B, C, Hi, Wi, p), dtype=torch.uint8, device="cuda")
    toks = torch.empty((cfg.B * (1 + N), cfg.D), dtype=dt, device="cuda")
    off = ctx.otas_patch_embed(_t(torch, imgs, dt), p, _t(torch, ends["w_patch"], dt), _t(torch, ends["b_patch"], dt),
                               _t(torch, ends["cls"], dt), _t(torch, ends["pos"], dt), ws, toks)
    torch.cuda.synchronize()
    assert off.tolist() == [q * (1 + N) for q in range(cfg.B + 1)]
    got = toks.to(torch.float32).cpu().numpy()
    for q in range(cfg.B):
        ref = orc.patch_embed(imgs[q], ends["w_patch"], ends["b_patch"], ends["cls"], ends["pos"], p, storage=st)
        assert hz.rel_err(got[off[q]:off[q + 1]], ref) <= tol, q
    # heads on a ragged float "encoder output"
    rng = np.random.default_rng(3)
    ns = [5, 1, 9]
    xoff = np.concatenate([[0], np.cumsum(ns)]).astype(np.int32)
    x = (rng.standard_normal((int(xoff[-1]), cfg.D)) * 3 + 0.5).astype(np.float32)
    task = [1, 0, 1]
    heads = [(_t(torch, ends[f"head_w{t}"], dt), _t(torch, ends[f"head_b{t}"], dt)) for t in range(2)]
    logits = torch.full((cfg.B, 40), float("nan"), dtype=torch.float32, device="cuda")
    ctx.otas_task_heads(_t(torch, x, torch.float32), xoff, task, heads, _t(torch, ends["lnf_g"], dt),
                        _t(torch, ends["lnf_b"], dt), logits)
    torch.cuda.synchronize()
    lg = logits.cpu().numpy()
    for q in range(cfg.B):
        t = task[q]
        ref = orc.task_head(x[xoff[q]:xoff[q + 1]].astype(np.float64), ends["lnf_g"], ends["lnf_b"],
                            ends[f"head_w{t}"], ends[f"head_b{t}"], cfg.ln_eps, storage=st)
        assert hz.rel_err(lg[q, :classes[t]], ref) <= tol, q
        assert np.all(lg[q, classes[t]:] == 0)
    # argument errors
    with pytest.raises(lib.OtasError) as e:      # image height not a multiple of the patch
        ctx.otas_patch_embed(_t(torch, imgs[:, :, :60], dt), p, _t(torch, ends["w_patch"], dt), _t(torch, ends["b_patch"], dt),
                             _t(torch, ends["cls"], dt), _t(torch, ends["pos"], dt), ws, toks)
    assert e.value.status == 1
    with pytest.raises(lib.OtasError) as e:      # task id out of range
        ctx.otas_task_heads(_t(torch, x, torch.float32), xoff, [0, 2, 1], heads, _t(torch, ends["lnf_g"], dt),
                            _t(torch, ends["lnf_b"], dt), logits)
    assert e.value.status == 1
    with pytest.raises(lib.OtasError) as e:      # head wider than the logits rows
        ctx.otas_task_heads(_t(torch, x, torch.float32), xoff, task, heads, _t(torch, ends["lnf_g"], dt),
                            _t(torch, ends["lnf_b"], dt), logits[:, :20].contiguous())
    assert e.value.status == 1
    ctx.close()


def test_image_to_logits_f32_with_prompts_and_merging(torch_cuda, lib):
    """The whole forward pass of the serving model (Sec. IV: inputs, tasks, task parameters, gamma):
    patch embedding -> prompt prepend -> token-adapted encoder -> task heads, fp32, against the oracle
    composed the same way; two queries of different tasks and strategies."""
    torch = torch_cuda
    cfg = synth.config("tiny")
    cfg.n0 = 1 + 14 * 14
    cfg.strategies = [(4, 8), (0, 16)]
    ctx, layers = hz.make_context(cfg)
    dt = ctx.torch_dtype
    C, Hi, Wi, p = 3, 224, 224, 16
    N = 196
    classes = [10, 100]
    ends = synth.ends_weights(cfg, C, p, N, classes)
    imgs = np.stack([synth.query_image(cfg, q, C, Hi, Wi) for q in range(2)])
    ws = torch.empty(ctx.otas_patch_embed_workspace_bytes(2, C, Hi, Wi, p), dtype=torch.uint8, device="cuda")
    toks = torch.empty((2 * (1 + N), cfg.D), dtype=dt, device="cuda")
    toff = ctx.otas_patch_embed(_t(torch, imgs, dt), p, _t(torch, ends["w_patch"], dt), _t(torch, ends["b_patch"], dt),
                                _t(torch, ends["cls"], dt), _t(torch, ends["pos"], dt), ws, toks)
    prm = [synth.query_prompts(cfg, q) for q in range(2)]
    prm_packed, prm_off = synth.pack(prm, cfg.D)
    x0 = torch.empty((int(toff[-1] + prm_off[-1]), cfg.D), dtype=dt, device="cuda")
    off = ctx.otas_prompt_prepend(toks, toff, _t(torch, prm_packed, dt), prm_off, x0)
    R = [8, 16]
    gpu = hz.gpu_forward(ctx, x0, off, R)
    x_packed = np.concatenate(gpu["x"], axis=0).astype(np.float32)
    heads = [(_t(torch, ends[f"head_w{t}"], dt), _t(torch, ends[f"head_b{t}"], dt)) for t in range(2)]
    logits = torch.zeros((2, 100), dtype=torch.float32, device="cuda")
    task = [0, 1]
    ctx.otas_task_heads(_t(torch, x_packed, torch.float32), gpu["offsets"], task, heads, _t(torch, ends["lnf_g"], dt),
                        _t(torch, ends["lnf_b"], dt), logits)
    torch.cuda.synchronize()
    lg = logits.cpu().numpy()
    for q in range(2):
        tk = orc.patch_embed(imgs[q], ends["w_patch"], ends["b_patch"], ends["cls"], ends["pos"], p)
        xq, _ = orc.prompt_prepend(tk, prm[q], cfg.n_lead)
        out = orc.encoder_forward_query(xq, layers, R[q], H=cfg.H, ln_eps=cfg.ln_eps, n_lead=cfg.n_lead)
        for l in range(cfg.L):
            assert np.array_equal(gpu["trace"][q][l][0], out["trace"][l][0]), (q, l)
        ref = orc.task_head(out["x"], ends["lnf_g"], ends["lnf_b"], ends[f"head_w{task[q]}"], ends[f"head_b{task[q]}"],
                            cfg.ln_eps)
        assert hz.rel_err(lg[q, :classes[task[q]]], ref) <= 1e-4, q
    ctx.close()


# ------------------------------------------------------------------------------------------- serving loop
def test_serving_engine_batches_match_oracle_and_loop_accounts(torch_cuda, lib):
    """The GPU engine of the serving loop (Sec. IV: a batch of inputs, their tasks, the task parameters and
    gamma in, per-task results out): one mixed-task batch per kind of gamma against the oracle composed the same
    way, then a short trace replayed through batching + token adaptation with every batch really executed."""
    torch = torch_cuda
    from paper_2401_05031_amd import serve
    cfg = synth.config("tiny")
    ctx, layers = hz.make_context(cfg)
    classes = (10, 100, 10)
    gammas = [-8, 0, 4]
    eng = serve.GpuEngine(ctx, cfg.n0, classes, max_prompts=4, pool=8, seed=3)
    toks = eng.tokens.float().cpu().numpy().reshape(8, cfg.n0, cfg.D)
    tasks = [2, 0, 1]
    for gi, g in enumerate(gammas):
        assert eng.run(tasks, gi, g) > 0.0
        lg = eng.logits[:3].cpu().numpy()
        P, r = serve.gamma_to_strategy(g)
        for q, task in enumerate(tasks):
            prm = eng.prompt_pool[task * eng.max_prompts:task * eng.max_prompts + P].float().cpu().numpy()
            xq, _ = orc.prompt_prepend(toks[q], prm, cfg.n_lead)
            out = orc.encoder_forward_query(xq, layers, r, H=cfg.H, ln_eps=cfg.ln_eps, n_lead=cfg.n_lead)
            w, b = eng.heads[task]
            ref = orc.task_head(out["x"], eng.lnf_g.float().cpu().numpy(), eng.lnf_b.float().cpu().numpy(),
                                w.float().cpu().numpy(), b.float().cpu().numpy(), cfg.ln_eps)
            assert hz.rel_err(lg[q, :classes[task]], ref) <= 1e-4, (g, q)
    lat = eng.measure_profile(gammas, 3, batch=8, repeats=3)
    assert (lat > 0).all()
    acc = synth.stand_in_accuracy(gammas, 3)
    thr0 = 1.0 / float(lat[:, 1].mean())
    scale = 580.0 / thr0
    trace = synth.poisson_trace(5, 3, time_scale=scale)
    sched = lib.Scheduler(gammas, lat, acc, serve.rate_table_from_latency(gammas, lat), delta=0.5 * scale,
                          eta=0.5 * scale, epsilon=8)
    res = serve.replay_trace(sched, trace, eng, acc, initial_stage=2.0 * scale, rate_window=scale, log=True)
    assert res["served"] + res["late"] + res["given_up"] == len(trace)
    assert res["batches"] > 0 and 0.0 < res["utility"] <= res["offered_utility"]
    assert sorted(i for rec in res["log"] for i in rec[2]) == list(range(len(trace)))
    assert all(len(rec[2]) <= 8 for rec in res["log"] if rec[0] == "run")
    ctx.close()


def test_many_short_queries_plan_larger_than_a_staging_slot(torch_cuda, lib):
    """6000 queries of 3 to 5 tokens: the per-call plan (offsets, merge counts and trace offsets per layer)
    is larger than one slot of the host staging ring, so the whole-buffer upload path runs; followed by an
    ordinary small call on the same context.  Sampled queries against the oracle, fp32."""
    cfg = synth.config("tiny")
    B = 6000
    rng = np.random.default_rng(17)
    n = rng.integers(3, 6, B)
    R = rng.integers(0, 3, B).tolist()
    base = synth.query_tokens(cfg, 0)
    toks = [np.ascontiguousarray(base[(7 * q) % 150:(7 * q) % 150 + n[q]]) for q in range(B)]
    prm = [np.zeros((0, cfg.D), dtype=np.float32)] * B
    ctx, layers = hz.make_context(cfg)
    x0, off = hz.gpu_prepend(ctx, toks, prm)
    gpu = hz.gpu_forward(ctx, x0, off, R, trace=False)
    for q in [0, 1, 2, 2999, 5998, 5999] + rng.integers(0, B, 10).tolist():
        ref = hz.oracle_forward(cfg, layers, [toks[q]], [prm[q]], [R[q]])
        assert gpu["x"][q].shape == ref[0]["x"].shape, q
        assert hz.rel_err(gpu["x"][q], ref[0]["x"]) <= F32_TOL, q
        assert np.array_equal(gpu["sizes"][q], ref[0]["sizes"]), q
    toks2, prm2, P2, R2 = synth.batch(cfg)
    x0, off = hz.gpu_prepend(ctx, toks2, prm2)
    gpu = hz.gpu_forward(ctx, x0, off, R2, trace=False)
    ref = hz.oracle_forward(cfg, layers, toks2, prm2, R2)
    for q in range(cfg.B):
        assert hz.rel_err(gpu["x"][q], ref[q]["x"]) <= F32_TOL
    ctx.close()


def test_clock_probe_samples_a_plausible_shader_clock(torch_cuda, lib):
    """The benchmark's shader-clock probe: every sample of a run on an idle GPU reads a clock between 0.3 and
    3 GHz, the samples agree with each other, a second probe reuses the buffer, a read without a probe is empty
    and bad sample counts are refused."""
    import paper_2401_05031_amd as otas
    cfg = synth.config("tiny")
    ctx, _ = hz.make_context(cfg)
    for n in (64, 200):
        ctx.otas_clock_probe_start(n)
        mhz = np.asarray(ctx.otas_clock_probe_read())
        assert mhz.shape == (n,)
        assert (mhz > 300).all() and (mhz < 3000).all(), (mhz.min(), mhz.max())
        body = mhz[n // 4:]
        assert body.max() - body.min() <= 0.2 * np.median(body)
    assert ctx.otas_clock_probe_read() == []
    for bad in (0, -1, otas.OTAS_CLOCK_PROBE_MAX_SAMPLES + 1):
        with pytest.raises(otas.OtasError):
            ctx.otas_clock_probe_start(bad)
    ctx.close()


def test_bench_prints_one_json_line_with_the_contract_keys(torch_cuda, lib):
    """bench.py as the driver runs it (a child process, few steps, a two-query oracle sample): exactly one
    JSON line on stdout with the agreed keys, a roofline object for the dominant kernel and the oracle baseline;
    more than one GPU is refused with a message."""
    import json
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--steps", "3", "--warmup", "1", "--others", "",
                        "--cpu-queries", "2", "--small-batches", "1,8"], capture_output=True, text=True, timeout=110,
                       cwd=root)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    b = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in b, k
    assert b["n_gpus"] == 1 and b["steps"] == 3 and b["warmup"] == 1 and b["higher_is_better"] is True
    assert b["unit"] == "images/s" and b["dtype"] == "bf16" and b["data"] == "synthetic" and b["vs_baseline"] is None
    assert "workload" in b["config"] and "model" not in b["config"]
    assert b["value"] == pytest.approx(64 / (b["ms_per_step"] * 1e-3), rel=1e-3)
    rf = b["roofline"]
    assert rf["bound"] == "mfma" and rf["unit"] == "TFLOP/s" and rf["peak"] == 2500.0
    assert rf["frac"] == pytest.approx(rf["achieved"] / rf["peak"], abs=1e-3) and 0.0 < rf["frac"] < 1.0
    assert rf["traffic"] is None or rf["traffic"] > 0
    # head width 64, bf16: attention and the merge plan of a layer go out as one launch, recorded as attention
    assert b["rooflines"]["attention"].get("includes_merge_plan") is True and "merge_plan" not in b["rooflines"]
    sm = b["small_batch_single_forward_ms_median"]
    assert set(sm) == {"1", "8"} and 0.0 < sm["1"] <= sm["8"] * 1.2 and sm["8"] < b["single_forward_ms_median"]
    sc = b["shader_clock"]
    assert 300 < sc["under_load_mhz"]["median"] <= sc["idle_mhz"] * 1.05 and sc["rated_mhz"] == 2400.0
    assert sc["peak_at_measured_clock"] == pytest.approx(2500.0 * sc["under_load_mhz"]["median"] / 2400.0, rel=1e-3)
    cb = b["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["unit"] == "images/s" and cb["value"] > 0 and cb["cores"] >= 1 and cb["sample"]
    r2 = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                        timeout=60, cwd=root)
    assert r2.returncode != 0 and "ONE GPU" in (r2.stderr + r2.stdout)
