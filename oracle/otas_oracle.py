"""CPU oracle for the token-adapted transformer encoder (OTAS, Sec. II-A/B/C and Sec. III-B).

TEST INFRASTRUCTURE ONLY.  This is a slow, plain float64 NumPy statement of what the method
computes, one query at a time, in the order the paper gives.  Only the tests, the smoke check and
the benchmark's cpu_baseline leg may import it; the HIP library never does and shares no code,
table or helper with it.

What each function follows
  * layer_norm, attention, mlp, encoder block order: Sec. II-A (normalisation, multi-head
    attention softmax(Q K^T / sqrt(d_k)) V with per-head projections, concatenation + linear,
    MLP) and Sec. III-B (prompting module before the normalisation, merging module before the
    MLP, both present in every layer; gamma = 0 is the unmodified transformer, Sec. III-D).
  * prompt_prepend: Sec. II-B / Sec. III-B (trained prompt tokens are concatenated in front of
    the input tokens; length n_i -> n_i + gamma).
  * merge_plan / merge_apply / token_merge: Sec. II-C (split the tokens into two sets, every
    token of set A picks its most similar token of set B, keep the |gamma| most similar edges,
    merge by weighted average, concatenate into a new sequence; length n_i -> n_i - |gamma|) with
    the similarity "obtained from multi-head attention" (Sec. III-B).

Readings taken where the paper is silent (each is also listed in the design notes):
  R1  sequence layout is [lead tokens | prompts | remaining tokens]; n_lead (0 or 1) leading
      tokens (the class token) are never merged away.
  R2  the two sets alternate by position: even positions -> A, odd positions -> B.
  R3  similarity = cosine similarity of the head-averaged attention keys of the same layer.
  R4  removal count per layer is r_eff = min(r, floor((n - n_lead)/2)).
  R5  ties: a row's best match is the lowest-index B token; edges of equal similarity are kept
      in order of lower A index first.
  R6  the new sequence keeps the surviving tokens in their original relative order.
  R7  the weighted average weights every token by the number of original tokens it stands for
      (its size); sizes add when tokens merge.
  R8  prompts are prepended once, before layer 0; merging happens in all L layers.
  R9  exact (erf) GELU, biased-variance LayerNorm with eps from the model description, biases on
      every Linear, no final norm and no head: the encoder is the stack of blocks.
  R10 optional size bias: + ln(size_j) on the logits of key j (not defined by the paper; off
      unless asked for; with all sizes 1 it changes nothing).
  R14 model ends (Sec. II-A vision transformer, Sec. III-B task heads): patches are taken row by
      row, flattened channel-major, projected linearly; [class token | patch tokens] + position
      embedding; the head of a query's task reads LayerNorm_final(first token).
  R13 per-layer prompting (Sec. III-B puts the prompting module in front of the normalisation
      of EVERY layer and counts gamma "per layer"; Sec. II-B speaks of prompts "added per layer"):
      two further readings next to R8, both only for queries that do not merge (Sec. III-B: a
      model performs either prompting or reduction during inference).  "replace": the P prompt
      rows of the sequence are overwritten with layer l's own trained prompts before the
      normalisation of every layer l >= 1, length constant n_i + P.  "grow": P new prompt rows
      are inserted in front of the input tokens (after the lead tokens, R1) before the
      normalisation of every layer l >= 1, length n_i + (l + 1) P.  Layer 0's prompts are the
      ones prompt_prepend put there.

Parity pins (tests/test_oracle_pins.py): gamma = 0 against torch.nn.TransformerEncoderLayer in
float64; length schedule closed forms; size conservation; size-weighted mean conservation;
brute-force edge selection on tiny inputs; closed-form tie cases; planted duplicate pairs;
identity cases; the merge metric (head-averaged keys of the same layer) and the merge's place in the
block (between the attention residual and the MLP) against an independent statement built from torch's
own block pieces, explicit loops and brute-force edges, with every misreading shown to differ; a
hand-worked head mean; a hand-worked edge_deficit case; per-layer prompting against the torch layer
applied block by block with the rows replaced / inserted by hand, closed forms with the residual
branches switched off, and the replacement of the prompt rows by their own values being a no-op.
No function here is without a pin.  The paper prints no worked numeric example for this path, so
nothing is pinned to a paper-printed value.

Storage modes.  storage="f64" computes everything in float64.  storage="bf16" keeps float64
arithmetic but rounds at the points where the HIP path of a bf16 model stores a tensor: to bf16
(float64 -> float32 -> bf16, ties to even) for the GEMM / attention operands -- LayerNorm output,
QKV, attention output, MLP hidden -- and to float32 for the residual stream (after each residual
add and after merging), which the HIP path keeps in float.  storage="f32" rounds to float32 at all
of these points.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
from scipy.special import erf as _erf

TINY_NORM = 1e-12


# ----------------------------------------------------------------------------- rounding
def round_storage(a: np.ndarray, storage: str) -> np.ndarray:
    """Round a float64 array to the storage type and return it as float64."""
    if storage == "f64":
        return a
    f = np.asarray(a, dtype=np.float64).astype(np.float32)
    if storage == "f32":
        return f.astype(np.float64)
    if storage == "bf16":
        bits = f.view(np.uint32).astype(np.uint64)
        lsb = (bits >> np.uint64(16)) & np.uint64(1)
        bits = (bits + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
        return bits.astype(np.uint32).view(np.float32).reshape(f.shape).astype(np.float64)
    raise ValueError(storage)


# ----------------------------------------------------------------------------- schedule
def removal_count(n: int, r: int, n_lead: int) -> int:
    """R4: tokens actually removed from a sequence of length n when r are asked for."""
    return max(0, min(int(r), (int(n) - int(n_lead)) // 2))


def length_schedule(n0: int, P: int, r: int, n_lead: int, L: int) -> List[int]:
    """Sequence length entering layer 0..L-1 and the output length (L+1 numbers).

    Sec. III-B shape laws: + P once (R8), then - r_eff in each of the L layers."""
    n = n0 + P
    out = [n]
    for _ in range(L):
        n -= removal_count(n, r, n_lead)
        out.append(n)
    return out


# ----------------------------------------------------------------------------- prompting
def prompt_prepend(tokens: np.ndarray, prompts: np.ndarray, n_lead: int) -> Tuple[np.ndarray, np.ndarray]:
    """Sec. II-B: put the P prompt rows in front of the input tokens (after the n_lead lead
    tokens, R1).  Returns the new sequence and sizes (all 1)."""
    tokens = np.asarray(tokens, dtype=np.float64)
    prompts = np.asarray(prompts, dtype=np.float64).reshape(-1, tokens.shape[1])
    x = np.concatenate([tokens[:n_lead], prompts, tokens[n_lead:]], axis=0)
    return x, np.ones(x.shape[0], dtype=np.int64)


def deep_length_schedule(n0: int, P: int, L: int, mode: str) -> List[int]:
    """R13: length entering layer 0..L-1 and the output length for per-layer prompting without
    merging: constant n0 + P ("replace"), or n0 + (l + 1) P entering layer l ("grow")."""
    if mode not in ("replace", "grow"):
        raise ValueError(mode)
    ent = [n0 + P * ((l + 1) if mode == "grow" else 1) for l in range(L)]
    return ent + [ent[-1] if L > 0 else n0 + P]


def deep_prompt_step(x: np.ndarray, sizes: np.ndarray, prompts: np.ndarray, n_lead: int, mode: str):
    """R13: the prompting module in front of layer l >= 1.  "replace": rows n_lead .. n_lead + P - 1
    take the values of this layer's prompts; "grow": the P prompts are inserted at row n_lead.
    Prompt rows stand for one token each (size 1)."""
    prompts = np.asarray(prompts, dtype=np.float64).reshape(-1, x.shape[1])
    P = prompts.shape[0]
    if mode == "replace":
        if n_lead + P > x.shape[0]:
            raise ValueError("more prompt rows than the sequence holds")
        x = x.copy()
        sizes = sizes.copy()
        x[n_lead:n_lead + P] = prompts
        sizes[n_lead:n_lead + P] = 1
        return x, sizes
    if mode == "grow":
        return (np.concatenate([x[:n_lead], prompts, x[n_lead:]], axis=0),
                np.concatenate([sizes[:n_lead], np.ones(P, dtype=sizes.dtype), sizes[n_lead:]]))
    raise ValueError(mode)


# ----------------------------------------------------------------------------- model ends
def patch_embed(image: np.ndarray, w_patch: np.ndarray, b_patch: np.ndarray, cls: Optional[np.ndarray],
                pos: np.ndarray, patch: int, storage: str = "f64") -> np.ndarray:
    """Sec. II-A (vision transformer): the image [C, Hi, Wi] is split into fixed-size patches (row
    by row, left to right), every patch is flattened (channel, then row, then column: the layout of
    a [D, C, p, p] projection weight) and projected linearly; the class token goes in front (if the
    model has one) and the position embedding pos[1 + N, D] (or [N, D] without class token) is added
    to every row.  Returns tokens [n_lead + N, D].  storage: where the HIP path stores a tensor
    (patch matrix, projection output, tokens) the value is rounded accordingly."""
    img = np.asarray(image, dtype=np.float64)
    C, Hi, Wi = img.shape
    p = int(patch)
    if Hi % p or Wi % p:
        raise ValueError("image size must be a multiple of the patch size")
    nh, nw = Hi // p, Wi // p
    rows = []
    for py in range(nh):
        for px in range(nw):
            rows.append(img[:, py * p:(py + 1) * p, px * p:(px + 1) * p].reshape(-1))
    pm = round_storage(np.stack(rows, axis=0), storage)                       # [N, C p p]
    W = np.asarray(w_patch, dtype=np.float64).reshape(-1, C * p * p)
    proj = round_storage(pm @ W.T + np.asarray(b_patch, dtype=np.float64), storage)
    pos = np.asarray(pos, dtype=np.float64)
    if cls is not None:
        seq = np.concatenate([np.asarray(cls, dtype=np.float64).reshape(1, -1), proj], axis=0)
    else:
        seq = proj
    if pos.shape != seq.shape:
        raise ValueError("position embedding must have one row per token")
    return round_storage(seq + pos, storage)


def task_head(x: np.ndarray, lnf_g: np.ndarray, lnf_b: np.ndarray, w_head: np.ndarray, b_head: np.ndarray,
              eps: float, storage: str = "f64") -> np.ndarray:
    """Sec. III-B / IV: every task has its own head parameters and a query is forwarded to the head of
    its task.  The head reads the first token of the encoder output (the class token) after a final
    LayerNorm (the vision transformer's, Sec. II-A): logits = W_task LN(x[0]) + b_task."""
    h = layer_norm(np.asarray(x, dtype=np.float64)[:1], np.asarray(lnf_g, dtype=np.float64),
                   np.asarray(lnf_b, dtype=np.float64), eps)
    h = round_storage(h, storage)
    return (h @ np.asarray(w_head, dtype=np.float64).T + np.asarray(b_head, dtype=np.float64))[0]


# ----------------------------------------------------------------------------- encoder pieces
def layer_norm(x: np.ndarray, g: np.ndarray, b: np.ndarray, eps: float) -> np.ndarray:
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g + b


def gelu(x: np.ndarray) -> np.ndarray:
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))


def softmax_rows(z: np.ndarray) -> np.ndarray:
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def qkv_project(h: np.ndarray, w_qkv: np.ndarray, b_qkv: np.ndarray) -> np.ndarray:
    """[n, 3D] = h W^T + b, columns ordered Q | K | V."""
    return h @ w_qkv.T + b_qkv


def attention_heads(qkv: np.ndarray, H: int, sizes: Optional[np.ndarray] = None,
                    size_bias: bool = False) -> np.ndarray:
    """Sec. II-A: per head softmax(Q_h K_h^T / sqrt(d_k)) V_h, heads concatenated -> [n, D]."""
    n, D3 = qkv.shape
    D = D3 // 3
    dh = D // H
    out = np.empty((n, D), dtype=np.float64)
    for h in range(H):
        Q = qkv[:, h * dh:(h + 1) * dh]
        K = qkv[:, D + h * dh:D + (h + 1) * dh]
        V = qkv[:, 2 * D + h * dh:2 * D + (h + 1) * dh]
        logits = (Q @ K.T) / math.sqrt(dh)
        if size_bias:
            logits = logits + np.log(np.asarray(sizes, dtype=np.float64))[None, :]
        out[:, h * dh:(h + 1) * dh] = softmax_rows(logits) @ V
    return out


def merge_metric_from_keys(qkv: np.ndarray, H: int) -> np.ndarray:
    """R3: per token, the mean over heads of its key vectors -> [n, d_h]."""
    n, D3 = qkv.shape
    D = D3 // 3
    dh = D // H
    return qkv[:, D:2 * D].reshape(n, H, dh).mean(axis=1)


# ----------------------------------------------------------------------------- merging
def merge_plan(metric: np.ndarray, r_eff: int, n_lead: int):
    """Sec. II-C steps 1-2.  metric [n, dm].  Returns (src, dst, info):
    src[k], dst[k] = positions (in the current sequence) of the k-th best kept edge, A token and
    its B token, in rank order; info carries the decision margins."""
    n = metric.shape[0]
    info = {"argmax_margin": math.inf, "rank_margin": math.inf, "sim": None, "best": None, "kth": math.inf}
    if r_eff <= 0:
        return np.zeros(0, dtype=np.int64), np.zeros(0, dtype=np.int64), info
    norm = np.sqrt((metric * metric).sum(axis=1, keepdims=True))
    mhat = metric / np.maximum(norm, TINY_NORM)
    a_pos = np.arange(0, n, 2)                      # set A: even positions (R2)
    b_pos = np.arange(1, n, 2)                      # set B: odd positions
    sim = mhat[a_pos] @ mhat[b_pos].T               # [|A|, |B|]
    sim[a_pos < n_lead, :] = -np.inf                # protected tokens never leave (R1)
    best_col = sim.argmax(axis=1)                   # first maximum = lowest B index (R5)
    best = sim[np.arange(a_pos.size), best_col]
    order = np.argsort(-best, kind="stable")        # descending, equal values: lower A first (R5)
    chosen = order[:r_eff]
    # decision margins, for the tests' robustness print-out and near-tie attribution
    info.update(sim=sim, best=best, kth=float(best[order[r_eff - 1]]))
    if sim.shape[1] > 1:
        part = np.sort(sim[chosen], axis=1)
        info["argmax_margin"] = float(np.min(part[:, -1] - part[:, -2]))
    if r_eff < a_pos.size:
        nxt = best[order[r_eff]]
        if np.isfinite(nxt):
            info["rank_margin"] = float(best[order[r_eff - 1]] - nxt)
    return a_pos[chosen], b_pos[best_col[chosen]], info


def edge_deficit(info: dict, a: int, b: int) -> float:
    """How far (in similarity) the edge (a, b) is from being one the oracle itself would keep:
    max(best[a] - sim[a,b], kth best - sim[a,b], 0).  0 for the oracle's own edges."""
    s = info["sim"][a // 2, b // 2]
    return float(max(info["best"][a // 2] - s, info["kth"] - s, 0.0))


def merge_apply(x: np.ndarray, sizes: np.ndarray, src: Sequence[int], dst: Sequence[int]):
    """Sec. II-C step 3 (R6, R7): size-weighted average of every merged A token into its B token,
    then drop the merged rows keeping the original order."""
    x = np.array(x, dtype=np.float64, copy=True)
    sizes = np.array(sizes, dtype=np.int64, copy=True)
    n = x.shape[0]
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    gone = np.zeros(n, dtype=bool)
    gone[src] = True
    for b in np.unique(dst):
        sources = np.sort(src[dst == b])            # ascending A position
        acc = sizes[b] * x[b]
        tot = int(sizes[b])
        for a in sources:
            acc = acc + sizes[a] * x[a]
            tot += int(sizes[a])
        x[b] = acc / tot
        sizes[b] = tot
    keep = ~gone
    return x[keep], sizes[keep]


def token_merge(x: np.ndarray, metric: np.ndarray, sizes: Optional[np.ndarray], r: int, n_lead: int):
    """One application of the merging module to one query.  Returns x', sizes', src, dst, info."""
    n = x.shape[0]
    if sizes is None:
        sizes = np.ones(n, dtype=np.int64)
    r_eff = removal_count(n, r, n_lead)
    src, dst, info = merge_plan(np.asarray(metric, dtype=np.float64), r_eff, n_lead)
    x2, s2 = merge_apply(x, sizes, src, dst)
    return x2, s2, src, dst, info


def validate_decision(n: int, r_eff: int, n_lead: int, src, dst) -> None:
    """Raise if (src, dst) is not a structurally valid set of r_eff merge edges for length n."""
    src = np.asarray(src)
    dst = np.asarray(dst)
    if src.shape != (r_eff,) or dst.shape != (r_eff,):
        raise ValueError(f"decision has {src.shape}/{dst.shape} edges, expected {r_eff}")
    if r_eff == 0:
        return
    if np.unique(src).size != r_eff:
        raise ValueError("a token is merged twice")
    if np.any(src % 2 != 0) or np.any(src < n_lead) or np.any(src >= n):
        raise ValueError("merge source outside the unprotected part of set A")
    if np.any(dst % 2 != 1) or np.any(dst >= n) or np.any(dst < 0):
        raise ValueError("merge destination outside set B")


# ----------------------------------------------------------------------------- whole encoder
def encoder_forward_query(x0: np.ndarray, layers: Sequence[Dict[str, np.ndarray]], r: int, *,
                          H: int, ln_eps: float, n_lead: int, storage: str = "f64",
                          size_bias: bool = False, adopt: Optional[Sequence] = None,
                          taps: Optional[dict] = None, sizes0: Optional[np.ndarray] = None,
                          deep_prompts: Optional[Sequence[Optional[np.ndarray]]] = None,
                          deep_mode: Optional[str] = None, arith: str = "f64"):
    """Token-adapted encoder for ONE query (prompts already prepended).

    arith: "f64" (the oracle proper) or "f32": the same steps with NumPy float32 arithmetic for the
    normalisations, linear layers, attention and the weighted average (merge decisions are still
    taken on float64 copies of the float32 metric).  Only the benchmark's second CPU figure uses it.

    deep_prompts / deep_mode (R13): per-layer prompting; deep_prompts[l] ([P, D]) is applied in
    front of layer l for l >= 1 (entry 0 is not used: layer 0's prompts are part of x0); needs
    r = 0 when any prompt row is given.

    adopt: optional per-layer (src, dst) decisions to apply instead of the oracle's own
    (lock-step comparison); the oracle still computes its own decision and reports how many edges
    differ and, for every adopted edge the oracle would not have kept, its similarity deficit
    (edge_deficit).  sizes0: sizes entering the first given layer (default all 1); taps: dict that
    receives per-layer intermediate states.  Returns dict(x, sizes, trace=[(src,dst) per layer],
    disagree=[per layer], margins=[per layer], lengths, deficits)."""
    if arith not in ("f64", "f32"):
        raise ValueError(arith)
    if arith == "f32":
        return _encoder_forward_query_f32(x0, layers, r, H=H, ln_eps=ln_eps, n_lead=n_lead, storage=storage,
                                          size_bias=size_bias)
    st = storage
    rs = "f32" if storage == "bf16" else storage          # storage of the residual stream
    x = round_storage(np.asarray(x0, dtype=np.float64), rs)
    n = x.shape[0]
    sizes = np.ones(n, dtype=np.int64) if sizes0 is None else np.array(sizes0, dtype=np.int64)
    trace, disagree, margins, lengths, deficits = [], [], [], [n], []
    if deep_prompts is not None:
        if deep_mode not in ("replace", "grow"):
            raise ValueError("deep_mode must be 'replace' or 'grow'")
        if r != 0 and any(p is not None and np.asarray(p).size for p in deep_prompts[1:]):
            raise ValueError("per-layer prompting is defined for queries that do not merge")
    for l, w in enumerate(layers):
        W = {k: np.asarray(v, dtype=np.float64) for k, v in w.items()}
        if deep_prompts is not None and l >= 1 and deep_prompts[l] is not None:
            # prompting module, in front of the normalisation (stored like the residual stream)
            x, sizes = deep_prompt_step(x, sizes, round_storage(np.asarray(deep_prompts[l], dtype=np.float64), rs),
                                        n_lead, deep_mode)
            if deep_mode == "grow":
                lengths[-1] = x.shape[0]
        if taps is not None:
            taps.setdefault("x_in", []).append(x.copy())
            taps.setdefault("sizes_in", []).append(sizes.copy())
        # normalisation -> multi-head attention -> residual
        h = round_storage(layer_norm(x, W["ln1_g"], W["ln1_b"], ln_eps), st)
        qkv = round_storage(qkv_project(h, W["w_qkv"], W["b_qkv"]), st)
        o = round_storage(attention_heads(qkv, H, sizes, size_bias), st)
        x = round_storage(x + o @ W["w_proj"].T + W["b_proj"], rs)
        if taps is not None:
            taps.setdefault("x_attn", []).append(x.copy())
            taps.setdefault("qkv", []).append(qkv.copy())
        # merging module, before the MLP
        r_eff = removal_count(x.shape[0], r, n_lead)
        metric = merge_metric_from_keys(qkv, H)
        src, dst, info = merge_plan(metric, r_eff, n_lead)
        n_dis = 0
        if adopt is not None:
            g_src, g_dst = (np.asarray(v, dtype=np.int64) for v in adopt[l])
            validate_decision(x.shape[0], r_eff, n_lead, g_src, g_dst)
            mine = set(zip(src.tolist(), dst.tolist()))
            theirs = set(zip(g_src.tolist(), g_dst.tolist()))
            n_dis = len(mine ^ theirs) // 2 + len(mine ^ theirs) % 2
            deficits.extend(edge_deficit(info, a, b) for a, b in theirs - mine)
            src, dst = g_src, g_dst
        if r_eff > 0:
            x, sizes = merge_apply(x, sizes, src, dst)
            x = round_storage(x, rs)
        trace.append((np.asarray(src), np.asarray(dst)))
        disagree.append(n_dis)
        margins.append({k: info[k] for k in ("argmax_margin", "rank_margin")})
        # normalisation -> MLP -> residual
        h2 = round_storage(layer_norm(x, W["ln2_g"], W["ln2_b"], ln_eps), st)
        hid = round_storage(gelu(h2 @ W["w_fc1"].T + W["b_fc1"]), st)
        x = round_storage(x + hid @ W["w_fc2"].T + W["b_fc2"], rs)
        lengths.append(x.shape[0])
        if taps is not None:
            taps.setdefault("x_out", []).append(x.copy())
    return {"x": x, "sizes": sizes, "trace": trace, "disagree": disagree,
            "margins": margins, "lengths": lengths, "deficits": deficits}


def _encoder_forward_query_f32(x0, layers, r, *, H, ln_eps, n_lead, storage, size_bias):
    """The block sequence of encoder_forward_query with float32 NumPy arithmetic (no lock-step, taps
    or per-layer prompting): normalisation -> attention -> residual -> merge -> normalisation -> MLP
    -> residual, rounding at the same storage points."""
    f = np.float32
    rs = "f32" if storage == "bf16" else storage

    def rnd(a, how):
        return round_storage(a, how).astype(f)

    x = rnd(np.asarray(x0, dtype=np.float64), rs)
    sizes = np.ones(x.shape[0], dtype=np.int64)
    trace, lengths = [], [x.shape[0]]
    for w in layers:
        W = {k: np.asarray(v, dtype=f) for k, v in w.items()}
        h = rnd(layer_norm(x, W["ln1_g"], W["ln1_b"], f(ln_eps)), storage)
        qkv = rnd(qkv_project(h, W["w_qkv"], W["b_qkv"]), storage)
        o = rnd(attention_heads(qkv, H, sizes, size_bias).astype(f), storage)
        x = rnd(x + o @ W["w_proj"].T + W["b_proj"], rs)
        r_eff = removal_count(x.shape[0], r, n_lead)
        src, dst, _ = merge_plan(merge_metric_from_keys(qkv, H).astype(np.float64), r_eff, n_lead)
        if r_eff > 0:
            x2, sizes = merge_apply(x, sizes, src, dst)
            x = rnd(x2, rs)
        trace.append((src, dst))
        h2 = rnd(layer_norm(x, W["ln2_g"], W["ln2_b"], f(ln_eps)), storage)
        hid = rnd(gelu(h2 @ W["w_fc1"].T + W["b_fc1"]).astype(f), storage)
        x = rnd(x + hid @ W["w_fc2"].T + W["b_fc2"], rs)
        lengths.append(x.shape[0])
    return {"x": x.astype(np.float64), "sizes": sizes, "trace": trace, "lengths": lengths}


def encoder_forward(x0_list: Sequence[np.ndarray], layers, r_list: Sequence[int], *, H: int,
                    ln_eps: float, n_lead: int, storage: str = "f64", size_bias: bool = False,
                    adopt: Optional[Sequence] = None):
    """A batch is a loop: queries never interact (Sec. III-B processes each sample's tokens)."""
    return [encoder_forward_query(x0, layers, r, H=H, ln_eps=ln_eps, n_lead=n_lead,
                                  storage=storage, size_bias=size_bias,
                                  adopt=None if adopt is None else adopt[q])
            for q, (x0, r) in enumerate(zip(x0_list, r_list))]
