"""Test harness: runs the same seeded workload through the HIP library (via the C ABI binding) and
through the CPU oracle, and compares.  Used by the GPU parity tests, the smoke check and the
benchmark's cpu_baseline leg; never by the library."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np

import otas_synth as synth
from oracle import otas_oracle as orc


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """The tolerance metric of the parity bars: max_i |got_i - ref_i| / max_i |ref_i| over one tensor
    (a max-norm relative error, NOT an element-wise one: element-wise relative error is meaningless
    at the zero crossings of a residual stream)."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30))


def elem_err(got: np.ndarray, ref: np.ndarray) -> float:
    """Element-wise companion of rel_err: max_i |got_i - ref_i| / max(|ref_i|, rms(ref)), i.e. the
    relative error of every element with the tensor's root mean square as the absolute floor (so an
    element near zero is held to an absolute error of bar * rms, a large one to bar * its size)."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    floor = max(float(np.sqrt(np.mean(ref * ref))), 1e-30)
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), floor)))


def storage_of(cfg: synth.Config) -> str:
    return "bf16" if cfg.dtype == "bf16" else "f64"


def make_context(cfg: synth.Config, layers_host: Optional[List[Dict[str, np.ndarray]]] = None):
    """Upload the synthetic weights and create the library context.  Returns (ctx, layers_host)."""
    import torch
    import paper_2401_05031_amd as otas
    if layers_host is None:
        layers_host = synth.all_weights(cfg)
    ctx = otas.Context.from_host_weights(cfg.L, cfg.D, cfg.H, cfg.F,
                                         otas.OTAS_F32 if cfg.dtype == "f32" else otas.OTAS_BF16,
                                         cfg.ln_eps, cfg.n_lead, layers_host)
    return ctx, layers_host


def gpu_prepend(ctx, toks: Sequence[np.ndarray], prm: Sequence[np.ndarray]):
    """otas_prompt_prepend on packed device tensors.  Returns (x0 device tensor, offsets)."""
    import torch
    D = ctx.D
    tok_packed, tok_off = synth.pack(toks, D)
    prm_packed, prm_off = synth.pack(prm, D)
    t_tok = torch.from_numpy(tok_packed).to("cuda").to(ctx.torch_dtype)
    t_prm = torch.from_numpy(prm_packed).to("cuda").to(ctx.torch_dtype) if prm_packed.shape[0] else None
    out = torch.empty((int(tok_off[-1] + prm_off[-1]), D), dtype=ctx.torch_dtype, device="cuda")
    out_off = ctx.otas_prompt_prepend(t_tok, tok_off, t_prm, prm_off, out)
    return out, out_off


def gpu_forward(ctx, x0, offsets, r: Sequence[int], flags: int = 0, trace: bool = True,
                layer_range=None, sizes_in=None):
    """otas_encoder_forward (or otas_encoder_layers when layer_range / sizes_in is given).  Returns
    dict with per-query outputs as float64 numpy arrays and, if trace, the per-query per-layer
    (src, dst) edges."""
    import torch
    import paper_2401_05031_amd as otas
    B = len(offsets) - 1
    T0 = int(offsets[-1])
    lengths0 = np.diff(np.asarray(offsets))
    l0, l1 = (0, ctx.L) if layer_range is None else layer_range
    nl = l1 - l0
    reff, troff = ctx.trace_layout(lengths0, r, nl)
    T_out = int(T0 - reff.sum())
    ws = torch.empty(ctx.otas_workspace_bytes(B, T0), dtype=torch.uint8, device="cuda")
    x_out = torch.empty((T_out, ctx.D), dtype=torch.float32, device="cuda")   # the residual stream is float
    sizes_out = torch.empty(T_out, dtype=torch.int32, device="cuda")
    n_tr = int(reff.sum())
    tsrc = torch.full((max(n_tr, 1),), -1, dtype=torch.int32, device="cuda")
    tdst = torch.full((max(n_tr, 1),), -1, dtype=torch.int32, device="cuda")
    if trace:
        flags |= otas.OTAS_FLAG_TRACE
    if layer_range is None and sizes_in is None:
        out_off = ctx.otas_encoder_forward(x0, offsets, r, flags, ws, x_out, sizes_out, tsrc, tdst)
    else:
        out_off = ctx.otas_encoder_layers(l0, l1, x0, sizes_in, offsets, r, flags, ws, x_out, sizes_out, tsrc, tdst)
    torch.cuda.synchronize()
    xo = x_out.to(torch.float32).cpu().numpy().astype(np.float64)
    so = sizes_out.cpu().numpy()
    res = {"x": [xo[out_off[q]:out_off[q + 1]] for q in range(B)],
           "sizes": [so[out_off[q]:out_off[q + 1]] for q in range(B)],
           "offsets": out_off, "T_out": T_out}
    if trace:
        hs, hd = tsrc.cpu().numpy(), tdst.cpu().numpy()
        res["trace"] = [[(hs[troff[l, q]:troff[l, q] + reff[l, q]], hd[troff[l, q]:troff[l, q] + reff[l, q]])
                         for l in range(nl)] for q in range(B)]
    return res


def oracle_forward(cfg: synth.Config, layers_host, toks, prm, r, adopt=None, size_bias: bool = False,
                   storage: Optional[str] = None):
    """The oracle on the same host arrays: prepend, then the encoder, one query at a time."""
    outs = []
    for q, (t, p) in enumerate(zip(toks, prm)):
        x0, _ = orc.prompt_prepend(t, p, cfg.n_lead)
        outs.append(orc.encoder_forward_query(
            x0, layers_host, r[q], H=cfg.H, ln_eps=cfg.ln_eps, n_lead=cfg.n_lead,
            storage=storage or storage_of(cfg), size_bias=size_bias,
            adopt=None if adopt is None else adopt[q]))
    return outs


def compare_lockstep(cfg, layers_host, toks, prm, r, gpu, size_bias: bool = False):
    """End to end, the oracle in lock-step with the GPU's merge decisions: it computes its own
    decision per layer, counts the edges that differ, records for each differing GPU edge how far
    (in oracle similarity) it is from an edge the oracle would keep, then applies the GPU's
    decision so that later layers stay comparable.  Returns dict(max_err, decisions,
    disagreements, max_deficit, sizes_equal)."""
    outs = oracle_forward(cfg, layers_host, toks, prm, r, adopt=gpu["trace"], size_bias=size_bias)
    max_err, dis, dec, sizes_equal, max_def, max_elem = 0.0, 0, 0, True, 0.0, 0.0
    for q, o in enumerate(outs):
        max_err = max(max_err, rel_err(gpu["x"][q], o["x"]))
        max_elem = max(max_elem, elem_err(gpu["x"][q], o["x"]))
        dis += int(sum(o["disagree"]))
        dec += int(sum(s.size for s, _ in o["trace"]))
        max_def = max([max_def] + o["deficits"])
        sizes_equal = sizes_equal and np.array_equal(gpu["sizes"][q], o["sizes"])
    return {"max_err": max_err, "elem_err": max_elem, "decisions": dec, "disagreements": dis,
            "max_deficit": max_def, "sizes_equal": sizes_equal}


def compare_per_layer(ctx, cfg, layers_host, toks, prm, r, size_bias: bool = False):
    """Layer by layer on identical inputs: the oracle runs freely (its own decisions) and records
    the state entering every block; the GPU then runs each block alone
    (otas_encoder_layers(l, l+1)) from the oracle's state, and its merge edges and output are
    compared with the oracle's for that block.  Data flows oracle -> GPU only.  Returns
    dict(decisions, disagreements, max_err, sizes_equal)."""
    import torch
    import paper_2401_05031_amd as otas
    taps = [dict() for _ in toks]
    outs = []
    for q, (t, p) in enumerate(zip(toks, prm)):
        x0, _ = orc.prompt_prepend(t, p, cfg.n_lead)
        outs.append(orc.encoder_forward_query(x0, layers_host, r[q], H=cfg.H, ln_eps=cfg.ln_eps,
                                              n_lead=cfg.n_lead, storage=storage_of(cfg),
                                              size_bias=size_bias, taps=taps[q]))
    dec = dis = 0
    max_err, max_elem, sizes_equal = 0.0, 0.0, True
    flags = otas.OTAS_FLAG_SIZE_BIAS if size_bias else 0
    for l in range(cfg.L):
        xs = [taps[q]["x_in"][l] for q in range(len(toks))]
        packed, off = synth.pack(xs, cfg.D)
        sz = np.concatenate([taps[q]["sizes_in"][l] for q in range(len(toks))]).astype(np.int32)
        x_d = torch.from_numpy(packed).to("cuda")               # float32: exactly the oracle's residual stream
        s_d = torch.from_numpy(sz).to("cuda")
        g = gpu_forward(ctx, x_d, off, r, flags=flags, layer_range=(l, l + 1), sizes_in=s_d)
        for q in range(len(toks)):
            src, dst = outs[q]["trace"][l]
            mine = set(zip(src.tolist(), dst.tolist()))
            theirs = set(zip(g["trace"][q][0][0].tolist(), g["trace"][q][0][1].tolist()))
            dec += len(mine)
            d = len(mine ^ theirs) // 2
            dis += d
            if d == 0:
                want_s = taps[q]["sizes_in"][l + 1] if l + 1 < cfg.L else outs[q]["sizes"]
                sizes_equal = sizes_equal and np.array_equal(g["sizes"][q], want_s)
                max_err = max(max_err, rel_err(g["x"][q], taps[q]["x_out"][l]))
                max_elem = max(max_elem, elem_err(g["x"][q], taps[q]["x_out"][l]))
    return {"decisions": dec, "disagreements": dis, "max_err": max_err, "elem_err": max_elem,
            "sizes_equal": sizes_equal}


def deep_prompt_tensor(cfg: synth.Config, queries: Sequence[int]):
    """Host array [L, sum P_q, D] of the per-layer prompts of the given queries (row block l = layer l's
    prompts of every query in order; block 0 repeats layer 0's prompts, which the library does not
    read) and the prompt offsets [len(queries) + 1]."""
    blocks = []
    for l in range(cfg.L):
        rows = [synth.query_prompts(cfg, q) if l == 0 else synth.query_layer_prompts(cfg, q, l) for q in queries]
        blocks.append(np.concatenate(rows, axis=0) if rows else np.zeros((0, cfg.D), dtype=np.float32))
    poff = np.concatenate([[0], np.cumsum([cfg.strategies[q][0] for q in queries])]).astype(np.int32)
    return np.stack(blocks, axis=0), poff


def gpu_forward_deep(ctx, cfg: synth.Config, queries: Sequence[int], mode: str):
    """otas_prompt_prepend + otas_encoder_forward_deep for the given queries.  Returns per-query
    outputs (float64) and the output offsets."""
    import torch
    import paper_2401_05031_amd as otas
    toks = [synth.query_tokens(cfg, q) for q in queries]
    prm0 = [synth.query_prompts(cfg, q) for q in queries]
    x0, off = gpu_prepend(ctx, toks, prm0)
    deep, poff = deep_prompt_tensor(cfg, queries)
    t_deep = torch.from_numpy(deep).to("cuda").to(ctx.torch_dtype).contiguous()
    grow = mode == "grow"
    T0 = int(off[-1])
    T_L = T0 + (cfg.L - 1) * int(poff[-1]) if grow else T0
    ws = torch.empty(ctx.otas_workspace_bytes(len(queries), T_L), dtype=torch.uint8, device="cuda")
    x_out = torch.full((T_L, cfg.D), float("nan"), dtype=torch.float32, device="cuda")
    sizes = torch.zeros(T_L, dtype=torch.int32, device="cuda")
    out_off = ctx.otas_encoder_forward_deep(x0, off, otas.OTAS_PROMPT_GROW if grow else otas.OTAS_PROMPT_REPLACE,
                                            t_deep if deep.shape[1] else None, poff, ws, x_out, sizes)
    torch.cuda.synchronize()
    xo = x_out.cpu().numpy().astype(np.float64)
    so = sizes.cpu().numpy()
    return {"x": [xo[out_off[i]:out_off[i + 1]] for i in range(len(queries))],
            "sizes": [so[out_off[i]:out_off[i + 1]] for i in range(len(queries))], "offsets": out_off}


def oracle_forward_deep(cfg: synth.Config, layers_host, queries: Sequence[int], mode: str):
    outs = []
    for q in queries:
        x0, _ = orc.prompt_prepend(synth.query_tokens(cfg, q), synth.query_prompts(cfg, q), cfg.n_lead)
        deep = [None] + [synth.query_layer_prompts(cfg, q, l) for l in range(1, cfg.L)]
        outs.append(orc.encoder_forward_query(x0, layers_host, 0, H=cfg.H, ln_eps=cfg.ln_eps, n_lead=cfg.n_lead,
                                              storage=storage_of(cfg), deep_prompts=deep, deep_mode=mode))
    return outs
