"""Seeded synthetic inputs for the token-adapted encoder (shapes of the paper's ViT workloads).

This module holds *no arithmetic of the method*: it only draws Gaussian tokens, prompts and
weights with the shapes the paper's experiment section fixes (ViT-Base/16: 12 layers, 12 heads,
width 768, 16x16 patches of a 224x224 image -> 1 CLS + 196 patch tokens) and the larger ViT
shapes used as stress cases.  Both the CPU oracle's tests and the HIP path's tests draw from
here, so the two sides see the same numbers; neither side's code lives here.

Every draw is keyed by (seed, stream tag, index) with a counter-style PCG64 seed sequence, so a
single query or a single layer can be regenerated without generating the rest (the large
configurations are checked on a subset of queries).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_TAG_TOKENS, _TAG_PROMPTS, _TAG_WEIGHTS, _TAG_STRATEGY, _TAG_LAYER_PROMPTS, _TAG_IMAGES, _TAG_ENDS = 1, 2, 3, 4, 5, 6, 7

WEIGHT_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_proj", "b_proj",
                "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


@dataclass
class Config:
    """One workload: model shape + batch + per-query token strategy (P prompts, r removals/layer)."""
    name: str
    L: int
    D: int
    H: int
    F: int
    dtype: str                    # "f32" or "bf16": the storage/compute type of the HIP path
    B: int
    n0: int                       # tokens per query before prompting (1 CLS + patches)
    strategies: List[Tuple[int, int]] = field(default_factory=list)   # per query (P, r)
    seed: int = 0
    ln_eps: float = 1e-6
    n_lead: int = 1               # protected leading tokens (the CLS token)
    deep: str = ""                # "", "replace" or "grow": per-layer prompting (r must be 0 then)

    @property
    def dh(self) -> int:
        return self.D // self.H


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16-representable float32 (ties to even).

    Input conditioning only: makes the generated numbers exactly representable in the 16-bit
    storage type so that the upload to the GPU is lossless.
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def _rng(seed: int, tag: int, index: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, tag, index])))


def _mixed_strategies(seed: int, B: int) -> List[Tuple[int, int]]:
    g = _rng(seed, _TAG_STRATEGY, 0)
    r = g.choice(np.array([0, 4, 8, 12]), size=B)
    p = g.choice(np.array([0, 10]), size=B)
    return [(int(pp), int(rr)) for pp, rr in zip(p, r)]


def config(name: str) -> Config:
    """The named workloads.  'tiny' is the fp32 parity case; the 'vitb_*' ones are the ViT-Base/16
    shape of the paper's experiment section at batch 64; 'vitl_ragged' and 'vith_mixed' are
    selective batches in which every query carries its own strategy."""
    if name == "tiny":
        return Config(name, L=2, D=192, H=3, F=768, dtype="f32", B=2, n0=197,
                      strategies=[(4, 8)] * 2, seed=0)
    if name == "vitb_plain":
        return Config(name, 12, 768, 12, 3072, "bf16", 64, 197, [(0, 0)] * 64, seed=1)
    if name == "vitb_r16":
        return Config(name, 12, 768, 12, 3072, "bf16", 64, 197, [(0, 16)] * 64, seed=1)
    if name == "vitb_p10_r8":
        return Config(name, 12, 768, 12, 3072, "bf16", 64, 197, [(10, 8)] * 64, seed=2)
    if name == "vitb_deep10_replace":   # ten prompt rows, re-written with every layer's own prompts
        return Config(name, 12, 768, 12, 3072, "bf16", 64, 197, [(10, 0)] * 64, seed=5, deep="replace")
    if name == "vitb_deep2_grow":       # two prompts added in front of every layer: 199, 201, ..., 221 rows
        return Config(name, 12, 768, 12, 3072, "bf16", 64, 197, [(2, 0)] * 64, seed=6, deep="grow")
    if name == "vitl_ragged":
        strat = [(10, 0)] * 32 + [(0, 8)] * 32 + [(0, 16)] * 32 + [(0, 24)] * 32
        return Config(name, 24, 1024, 16, 4096, "bf16", 128, 197, strat, seed=3)
    if name == "vith_mixed":
        return Config(name, 32, 1280, 16, 5120, "bf16", 256, 257, _mixed_strategies(4, 256), seed=4)
    raise KeyError(name)


CONFIG_NAMES = ("tiny", "vitb_plain", "vitb_r16", "vitb_p10_r8", "vitl_ragged", "vith_mixed",
                "vitb_deep10_replace", "vitb_deep2_grow")


def _maybe_round(a: np.ndarray, dtype: str) -> np.ndarray:
    return round_to_bf16(a) if dtype == "bf16" else a.astype(np.float32)


def query_tokens(cfg: Config, q: int) -> np.ndarray:
    """[n0, D] float32 token embeddings of query q, i.i.d. N(0,1)."""
    return _maybe_round(_rng(cfg.seed, _TAG_TOKENS, q).standard_normal((cfg.n0, cfg.D)), cfg.dtype)


def query_prompts(cfg: Config, q: int) -> np.ndarray:
    """[P_q, D] float32 prompt rows of query q, i.i.d. N(0, std 0.02)."""
    P = cfg.strategies[q][0]
    return _maybe_round(0.02 * _rng(cfg.seed, _TAG_PROMPTS, q).standard_normal((P, cfg.D)), cfg.dtype)


def query_layer_prompts(cfg: Config, q: int, l: int) -> np.ndarray:
    """[P_q, D] float32 prompt rows of query q for layer l >= 1 (per-layer prompting; layer 0's rows
    are query_prompts), i.i.d. N(0, std 0.02)."""
    P = cfg.strategies[q][0]
    g = _rng(cfg.seed, _TAG_LAYER_PROMPTS, q * 4096 + l)
    return _maybe_round(0.02 * g.standard_normal((P, cfg.D)), cfg.dtype)


def query_image(cfg: Config, q: int, C: int, Hi: int, Wi: int) -> np.ndarray:
    """[C, Hi, Wi] float32 image of query q, i.i.d. N(0,1) (stands in for a normalised picture)."""
    return _maybe_round(_rng(cfg.seed, _TAG_IMAGES, q).standard_normal((C, Hi, Wi)), cfg.dtype)


def ends_weights(cfg: Config, C: int, patch: int, n_patches: int, classes: Sequence[int]) -> Dict[str, np.ndarray]:
    """Parameters of the model ends: patch projection [D, C p p] + bias, class token, position
    embedding [n_lead + N, D], final LayerNorm, one head [K_t, D] + bias per task; N(0, std 0.02),
    LayerNorm scale 1, shift 0."""
    g = _rng(cfg.seed, _TAG_ENDS, 0)
    D = cfg.D
    w = {"w_patch": 0.02 * g.standard_normal((D, C * patch * patch)), "b_patch": 0.02 * g.standard_normal(D),
         "cls": 0.02 * g.standard_normal(D), "pos": 0.02 * g.standard_normal((cfg.n_lead + n_patches, D)),
         "lnf_g": np.ones(D), "lnf_b": np.zeros(D)}
    for t, K in enumerate(classes):
        w[f"head_w{t}"] = 0.02 * g.standard_normal((K, D))
        w[f"head_b{t}"] = 0.02 * g.standard_normal(K)
    return {k: _maybe_round(v, cfg.dtype) for k, v in w.items()}


def layer_weights(cfg: Config, l: int) -> Dict[str, np.ndarray]:
    """Weights of encoder block l.  Linear weights are [out, in]; every Linear weight and bias is
    N(0, std 0.02); LayerNorm scale 1, shift 0.  w_qkv rows are ordered Q | K | V with the heads
    contiguous inside each third."""
    g = _rng(cfg.seed, _TAG_WEIGHTS, l)
    D, F = cfg.D, cfg.F
    w = {
        "ln1_g": np.ones(D), "ln1_b": np.zeros(D),
        "w_qkv": 0.02 * g.standard_normal((3 * D, D)), "b_qkv": 0.02 * g.standard_normal(3 * D),
        "w_proj": 0.02 * g.standard_normal((D, D)), "b_proj": 0.02 * g.standard_normal(D),
        "ln2_g": np.ones(D), "ln2_b": np.zeros(D),
        "w_fc1": 0.02 * g.standard_normal((F, D)), "b_fc1": 0.02 * g.standard_normal(F),
        "w_fc2": 0.02 * g.standard_normal((D, F)), "b_fc2": 0.02 * g.standard_normal(D),
    }
    return {k: _maybe_round(v, cfg.dtype) for k, v in w.items()}


def all_weights(cfg: Config) -> List[Dict[str, np.ndarray]]:
    return [layer_weights(cfg, l) for l in range(cfg.L)]


def batch(cfg: Config, queries: Optional[Sequence[int]] = None):
    """Tokens, prompts and strategies of the selected queries (default: all).

    Returns (tokens list of [n0,D], prompts list of [P_q,D], P list, r list)."""
    qs = list(range(cfg.B)) if queries is None else list(queries)
    toks = [query_tokens(cfg, q) for q in qs]
    prm = [query_prompts(cfg, q) for q in qs]
    return toks, prm, [cfg.strategies[q][0] for q in qs], [cfg.strategies[q][1] for q in qs]


def pack(rows: Sequence[np.ndarray], D: int):
    """Concatenate per-query [n_q, D] arrays into one packed [T, D] array + offsets[B+1]."""
    offs = np.zeros(len(rows) + 1, dtype=np.int32)
    for i, a in enumerate(rows):
        offs[i + 1] = offs[i] + a.shape[0]
    if len(rows) == 0:
        return np.zeros((0, D), dtype=np.float32), offs
    return np.concatenate([np.asarray(a, dtype=np.float32).reshape(-1, D) for a in rows], axis=0), offs


# ------------------------------------------------------------------------------------------ serving traces
# Query types of the paper's synthetic trace (Table II): (task, latency requirement in s, utility).  Tasks 0, 1, 2
# stand for the three data sets of the experiment.
QUERY_TYPES: Tuple[Tuple[int, float, float], ...] = ((0, 0.6, 0.3), (0, 1.0, 0.01), (1, 0.6, 1.0), (1, 1.0, 0.2),
                                                     (2, 0.6, 0.3), (2, 1.0, 0.01))
GAMMA_LIST: Tuple[int, ...] = (-20, -15, -10, -5, 0, 2, 4, 8)      # selection list of the experiment (Sec. V)
TASK_CLASSES: Tuple[int, ...] = (10, 100, 10)                      # classes of the three tasks' heads


def poisson_trace(seed: int, seconds: int, rate_lo: float = 200.0, rate_hi: float = 700.0,
                  time_scale: float = 1.0) -> List[Tuple[float, float, float, int]]:
    """Synthetic query trace shaped like the paper's (Sec. V, workloads): in every second the request rate is
    drawn uniformly from [rate_lo, rate_hi] and arrivals within the second are a Poisson process of that rate;
    each request takes one of the six query types uniformly.  Returns rows (s_r, l_r, u_r, task) in arrival
    order.  time_scale < 1 compresses the clock (arrival times AND latency requirements) so that a faster
    device sees the same load relative to its capacity; rates scale by 1 / time_scale."""
    rng = np.random.default_rng([seed, 0x7A])
    rows = []
    for sec in range(seconds):
        rate = rng.uniform(rate_lo, rate_hi)
        t = float(sec)
        while True:
            t += rng.exponential(1.0 / rate)
            if t >= sec + 1:
                break
            task, lat, u = QUERY_TYPES[int(rng.integers(len(QUERY_TYPES)))]
            rows.append((t * time_scale, lat * time_scale, u, task))
    return rows


def stand_in_accuracy(gammas: Sequence[int] = GAMMA_LIST, n_tasks: int = 3) -> np.ndarray:
    """[n_tasks][len(gammas)] accuracy table standing in for the paper's profiled accuracies, which need its
    data sets and trained prompts.  Shaped like what the paper reports for token merging (Sec. II-C): a slight
    loss down to 15 merged tokens per layer, a sharp one beyond, roughly halving the accuracy at 25; prompts
    add a little, saturating.  Offset and scaled per task.  The shape, not the values, is what the scheduler
    needs."""
    base = np.array([0.97, 0.88, 0.95])[:n_tasks, None]
    g = np.asarray(gammas, dtype=np.float64)[None, :]
    m = np.maximum(-g, 0.0)
    drop = np.where(g < 0, 0.0015 * m + 0.0043 * np.maximum(m - 15.0, 0.0) ** 2, -0.012 * (1.0 - np.exp(-g / 4.0)))
    return np.clip(base - drop * (1.0 + 0.5 * np.arange(n_tasks)[:, None]), 0.0, 1.0)
