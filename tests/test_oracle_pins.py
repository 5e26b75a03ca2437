"""Pins for the CPU oracle: each test ties one part of oracle/otas_oracle.py to something other
than itself — an independent library routine, a closed form, an invariant of the method, or a
brute-force enumeration — so that a dropped term, a wrong sign or index, or a transposed operand
fails at least one of them.  CPU only."""
import itertools
import math

import numpy as np
import pytest
import torch

import otas_synth as synth
from oracle import otas_oracle as orc


def _rand_layers(rng, L, D, F, scale=0.2):
    out = []
    for _ in range(L):
        out.append({
            "ln1_g": 1 + 0.1 * rng.standard_normal(D), "ln1_b": 0.1 * rng.standard_normal(D),
            "w_qkv": scale * rng.standard_normal((3 * D, D)), "b_qkv": scale * rng.standard_normal(3 * D),
            "w_proj": scale * rng.standard_normal((D, D)), "b_proj": scale * rng.standard_normal(D),
            "ln2_g": 1 + 0.1 * rng.standard_normal(D), "ln2_b": 0.1 * rng.standard_normal(D),
            "w_fc1": scale * rng.standard_normal((F, D)), "b_fc1": scale * rng.standard_normal(F),
            "w_fc2": scale * rng.standard_normal((D, F)), "b_fc2": scale * rng.standard_normal(D),
        })
    return out


# ------------------------------------------------------------------ gamma = 0 is the plain encoder
def _torch_encoder(layers, D, H, F, eps):
    mods = []
    for w in layers:
        m = torch.nn.TransformerEncoderLayer(D, H, F, dropout=0.0, activation="gelu",
                                             layer_norm_eps=eps, batch_first=True, norm_first=True,
                                             dtype=torch.float64)
        sd = {
            "self_attn.in_proj_weight": w["w_qkv"], "self_attn.in_proj_bias": w["b_qkv"],
            "self_attn.out_proj.weight": w["w_proj"], "self_attn.out_proj.bias": w["b_proj"],
            "linear1.weight": w["w_fc1"], "linear1.bias": w["b_fc1"],
            "linear2.weight": w["w_fc2"], "linear2.bias": w["b_fc2"],
            "norm1.weight": w["ln1_g"], "norm1.bias": w["ln1_b"],
            "norm2.weight": w["ln2_g"], "norm2.bias": w["ln2_b"],
        }
        m.load_state_dict({k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in sd.items()})
        mods.append(m.eval())
    return mods


# ------------------------------------------------------------------ per-layer prompting (R13)
@pytest.mark.parametrize("mode", ["replace", "grow"])
@pytest.mark.parametrize("n_lead", [0, 1])
def test_per_layer_prompting_against_library_blocks(mode, n_lead):
    """Sec. III-B: the prompting module sits in front of every layer's normalisation.  Independent
    statement: torch's own encoder layer applied block by block, with the prompt rows overwritten /
    inserted by hand (torch tensor surgery) between the blocks."""
    rng = np.random.default_rng(11)
    n0, P, D, H, F, L = 9, 3, 16, 2, 32, 4
    layers = _rand_layers(rng, L, D, F)
    toks = rng.standard_normal((n0, D))
    prm = [rng.standard_normal((P, D)) for _ in range(L)]
    x0, _ = orc.prompt_prepend(toks, prm[0], n_lead)
    got = orc.encoder_forward_query(x0, layers, 0, H=H, ln_eps=1e-6, n_lead=n_lead,
                                    deep_prompts=prm, deep_mode=mode)
    with torch.no_grad():
        t = torch.from_numpy(x0)[None]
        for l, m in enumerate(_torch_encoder(layers, D, H, F, 1e-6)):
            if l >= 1:
                pl = torch.from_numpy(prm[l])[None]
                if mode == "replace":
                    t = torch.cat([t[:, :n_lead], pl, t[:, n_lead + P:]], dim=1)
                else:
                    t = torch.cat([t[:, :n_lead], pl, t[:, n_lead:]], dim=1)
            t = m(t)
    ref = t[0].numpy()
    assert got["x"].shape == ref.shape == (orc.deep_length_schedule(n0, P, L, mode)[-1], D)
    assert np.max(np.abs(got["x"] - ref)) <= 1e-11 * max(1.0, np.max(np.abs(ref)))
    assert got["lengths"] == orc.deep_length_schedule(n0, P, L, mode)
    assert got["sizes"].tolist() == [1] * ref.shape[0]


def test_per_layer_prompting_closed_forms_and_noop():
    """With both residual branches switched off (projection and second MLP linear zero) a block is
    the identity, so the output is known in closed form: "replace" leaves the last layer's prompts
    in the prompt rows, "grow" stacks the layers' prompts newest first in front of the tokens.
    Replacing the prompt rows by the values they already hold changes nothing; one layer has no
    per-layer step at all; merging together with per-layer prompts is refused."""
    rng = np.random.default_rng(12)
    n0, P, D, H, F, L = 7, 2, 8, 2, 16, 3
    layers = _rand_layers(rng, L, D, F)
    toks = rng.standard_normal((n0, D))
    prm = [rng.standard_normal((P, D)) for _ in range(L)]
    x0, _ = orc.prompt_prepend(toks, prm[0], 1)
    off = [dict(w, w_proj=np.zeros((D, D)), b_proj=np.zeros(D), w_fc2=np.zeros((D, F)), b_fc2=np.zeros(D)) for w in layers]
    rep = orc.encoder_forward_query(x0, off, 0, H=H, ln_eps=1e-6, n_lead=1, deep_prompts=prm, deep_mode="replace")
    assert np.array_equal(rep["x"], np.concatenate([toks[:1], prm[L - 1], toks[1:]]))
    grw = orc.encoder_forward_query(x0, off, 0, H=H, ln_eps=1e-6, n_lead=1, deep_prompts=prm, deep_mode="grow")
    assert np.array_equal(grw["x"], np.concatenate([toks[:1]] + [prm[l] for l in range(L - 1, -1, -1)] + [toks[1:]]))
    assert orc.deep_length_schedule(n0, P, L, "grow") == [n0 + P, n0 + 2 * P, n0 + 3 * P, n0 + 3 * P]
    assert orc.deep_length_schedule(n0, P, L, "replace") == [n0 + P] * (L + 1)
    # replacing the prompt rows with what they hold is a no-op
    taps = {}
    plain = orc.encoder_forward_query(x0, layers, 0, H=H, ln_eps=1e-6, n_lead=1, taps=taps)
    same = [None] + [taps["x_in"][l][1:1 + P] for l in range(1, L)]
    again = orc.encoder_forward_query(x0, layers, 0, H=H, ln_eps=1e-6, n_lead=1, deep_prompts=same, deep_mode="replace")
    assert np.array_equal(again["x"], plain["x"])
    # no prompt rows: both modes are the plain encoder
    none = [np.zeros((0, D))] * L
    for mode in ("replace", "grow"):
        z = orc.encoder_forward_query(x0, layers, 0, H=H, ln_eps=1e-6, n_lead=1, deep_prompts=none, deep_mode=mode)
        assert np.array_equal(z["x"], plain["x"])
    # a single layer has no per-layer step
    one = orc.encoder_forward_query(x0, layers[:1], 0, H=H, ln_eps=1e-6, n_lead=1, deep_prompts=prm[:1], deep_mode="grow")
    assert np.array_equal(one["x"], orc.encoder_forward_query(x0, layers[:1], 0, H=H, ln_eps=1e-6, n_lead=1)["x"])
    with pytest.raises(ValueError):
        orc.encoder_forward_query(x0, layers, 2, H=H, ln_eps=1e-6, n_lead=1, deep_prompts=prm, deep_mode="replace")
    with pytest.raises(ValueError):
        orc.encoder_forward_query(x0, layers, 0, H=H, ln_eps=1e-6, n_lead=1, deep_prompts=prm, deep_mode="append")


@pytest.mark.parametrize("n,D,H,F,L", [(7, 16, 2, 32, 2), (33, 48, 3, 96, 3)])
def test_gamma_zero_equals_library_prenorm_encoder(n, D, H, F, L):
    """Sec. III-D: gamma = 0 is the unmodified transformer.  The independent implementation is
    torch.nn.TransformerEncoderLayer (norm_first, exact GELU) in float64."""
    rng = np.random.default_rng(5)
    layers = _rand_layers(rng, L, D, F)
    x0 = rng.standard_normal((n, D))
    got = orc.encoder_forward_query(x0, layers, 0, H=H, ln_eps=1e-6, n_lead=1)
    # the fused fast path of the torch layer is inference-only and needs no_grad; both paths agree
    with torch.no_grad():
        t = torch.from_numpy(x0)[None]
        for m in _torch_encoder(layers, D, H, F, 1e-6):
            t = m(t)
    ref = t[0].numpy()
    assert got["x"].shape == (n, D)
    assert np.max(np.abs(got["x"] - ref)) <= 1e-11 * max(1.0, np.max(np.abs(ref)))
    assert got["sizes"].tolist() == [1] * n
    assert all(s.size == 0 for s, _ in got["trace"])


def test_attention_matches_library_sdpa_and_rows_sum_to_one():
    rng = np.random.default_rng(1)
    n, H, dh = 19, 4, 8
    qkv = rng.standard_normal((n, 3 * H * dh))
    got = orc.attention_heads(qkv, H)
    t = torch.from_numpy(qkv)
    q, k, v = (t[:, i * H * dh:(i + 1) * H * dh].reshape(n, H, dh).transpose(0, 1) for i in range(3))
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v).transpose(0, 1).reshape(n, H * dh)
    assert np.allclose(got, ref.numpy(), rtol=0, atol=1e-12)
    z = rng.standard_normal((5, 11)) * 30
    assert np.allclose(orc.softmax_rows(z).sum(axis=1), 1.0, atol=1e-14)


def test_layer_norm_and_gelu_match_library_and_closed_form():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((6, 40)) * 3 + 1
    g, b = rng.standard_normal(40), rng.standard_normal(40)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (40,), torch.from_numpy(g), torch.from_numpy(b), 1e-6)
    assert np.allclose(orc.layer_norm(x, g, b, 1e-6), ref.numpy(), atol=1e-12)
    v = np.linspace(-6, 6, 101)
    closed = np.array([0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in v])
    assert np.allclose(orc.gelu(v), closed, atol=1e-15)
    assert orc.gelu(np.array([0.0]))[0] == 0.0
    assert abs(orc.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15   # Phi(1)


def test_bf16_rounding_matches_library_cast():
    rng = np.random.default_rng(3)
    a = np.concatenate([rng.standard_normal(5000) * 10.0 ** rng.integers(-6, 6, 5000),
                        np.array([1.00390625, 1.01171875, 0.0, -0.0, 65280.0])])  # exact ties: to even
    ref = torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(orc.round_storage(a, "bf16"), ref)
    assert np.array_equal(synth.round_to_bf16(a.astype(np.float32)).astype(np.float64), ref)
    assert orc.round_storage(np.array([1.00390625]), "bf16")[0] == 1.0          # tie -> even mantissa
    assert orc.round_storage(np.array([1.01171875]), "bf16")[0] == 1.015625


# ------------------------------------------------------------------ shape laws / schedule
def test_length_schedule_closed_forms():
    """Sec. III-B: n_i + gamma after prompting, n_i - |gamma| after each merging module."""
    assert orc.length_schedule(197, 4, 8, 1, 2) == [201, 193, 185]
    assert orc.length_schedule(197, 0, 0, 1, 12) == [197] * 13
    assert orc.length_schedule(197, 0, 16, 1, 12) == [197 - 16 * i for i in range(12)] + [11]
    assert orc.length_schedule(197, 10, 8, 1, 12) == [207 - 8 * i for i in range(13)]
    # r = 24 collapses to the floor of two tokens (class token + one)
    s = orc.length_schedule(197, 0, 24, 1, 24)
    assert s[:14] == [197, 173, 149, 125, 101, 77, 53, 29, 15, 8, 5, 3, 2, 2] and set(s[14:]) == {2}
    # no protected token: floor is one token
    assert orc.length_schedule(8, 0, 100, 0, 5) == [8, 4, 2, 1, 1, 1]
    for n, r, nl in itertools.product(range(1, 40), range(0, 30), (0, 1)):
        if n < nl + 1:
            continue
        k = orc.removal_count(n, r, nl)
        assert 0 <= k <= r and n - k >= nl + (1 if n > nl else 0)
        assert k <= n // 2                       # never more edges than set B has tokens


def test_prompt_prepend_layout_and_identity():
    rng = np.random.default_rng(0)
    tok = rng.standard_normal((6, 4))
    pr = rng.standard_normal((3, 4))
    x, s = orc.prompt_prepend(tok, pr, 1)
    assert x.shape == (9, 4) and s.tolist() == [1] * 9
    assert np.array_equal(x[0], tok[0]) and np.array_equal(x[1:4], pr) and np.array_equal(x[4:], tok[1:])
    x0, _ = orc.prompt_prepend(tok, pr, 0)
    assert np.array_equal(x0[:3], pr) and np.array_equal(x0[3:], tok)
    xi, _ = orc.prompt_prepend(tok, np.zeros((0, 4)), 1)
    assert np.array_equal(xi, tok)


# ------------------------------------------------------------------ merge selection
def _brute_force_edges(metric, r_eff, n_lead):
    """Independent statement of Sec. II-C steps 1-2 with explicit Python loops and a full sort of
    explicit edge records (no argmax / argsort on matrices)."""
    n = metric.shape[0]
    unit = []
    for i in range(n):
        nrm = math.sqrt(sum(float(v) * float(v) for v in metric[i]))
        unit.append([float(v) / max(nrm, 1e-12) for v in metric[i]])
    picks = []
    for a in range(0, n, 2):
        if a < n_lead:
            continue
        edges = []
        for b in range(1, n, 2):
            edges.append((-sum(p * q for p, q in zip(unit[a], unit[b])), b))
        edges.sort()
        picks.append((edges[0][0], a, edges[0][1]))      # (-similarity, a, b)
    picks.sort()
    return [(a, b) for _, a, b in picks[:r_eff]]


@pytest.mark.parametrize("n_lead", [0, 1])
def test_merge_selection_matches_brute_force(n_lead):
    rng = np.random.default_rng(11)
    for n in range(2, 13):
        for trial in range(6):
            metric = rng.standard_normal((n, 5))
            if trial % 2:                               # signed one-hot rows: cosines are exactly
                metric = np.zeros((n, 5))               # -1, 0 or 1 on both sides -> many exact ties
                metric[np.arange(n), rng.integers(0, 3, n)] = rng.choice([-1.0, 1.0, 2.0, 4.0], n)
            for r in range(0, n):
                r_eff = orc.removal_count(n, r, n_lead)
                src, dst, _ = orc.merge_plan(metric, r_eff, n_lead)
                want = _brute_force_edges(metric, r_eff, n_lead)
                assert list(zip(src.tolist(), dst.tolist())) == want, (n, r, n_lead, trial)
                orc.validate_decision(n, r_eff, n_lead, src, dst)


def test_tie_rules_closed_form():
    """All tokens identical: every similarity is equal, so every A token picks the first B token
    (position 1) and the merged set is the r lowest unprotected even positions, in order."""
    x = np.tile(np.array([[0.5, -1.0, 2.0, 0.25]]), (11, 1))
    src, dst, _ = orc.merge_plan(x, 3, 1)
    assert src.tolist() == [2, 4, 6] and dst.tolist() == [1, 1, 1]
    src, dst, _ = orc.merge_plan(x, 3, 0)
    assert src.tolist() == [0, 2, 4] and dst.tolist() == [1, 1, 1]
    x2, s2, *_ = orc.token_merge(x, x, None, 3, 1)
    assert x2.shape[0] == 8 and s2.tolist() == [1, 4, 1, 1, 1, 1, 1, 1]
    assert np.allclose(x2, x[:8], atol=1e-15)


def test_planted_duplicate_pairs_are_the_merged_edges():
    rng = np.random.default_rng(4)
    n, d, r = 41, 16, 5
    x = rng.standard_normal((n, d))
    ks = [1, 4, 7, 12, 19]
    for k in ks:
        x[2 * k + 1] = x[2 * k] * 1.0                   # exact duplicates: cosine is exactly the row max
    x2, s2, src, dst, _ = orc.token_merge(x, x, None, r, 1)
    assert sorted(zip(src.tolist(), dst.tolist())) == [(2 * k, 2 * k + 1) for k in ks]
    assert x2.shape[0] == n - r
    kept = [i for i in range(n) if i not in {2 * k for k in ks}]
    for j, i in enumerate(kept):
        if i in {2 * k + 1 for k in ks}:
            assert s2[j] == 2 and np.allclose(x2[j], x[i], atol=1e-15)
        else:
            assert s2[j] == 1 and np.array_equal(x2[j], x[i])


def test_scaled_metric_rows_do_not_change_the_decision():
    """Cosine similarity: rescaling any token's metric vector by a positive factor changes nothing."""
    rng = np.random.default_rng(8)
    m = rng.standard_normal((30, 12))
    a = orc.merge_plan(m, 7, 1)
    b = orc.merge_plan(m * rng.uniform(0.1, 9.0, size=(30, 1)), 7, 1)
    assert a[0].tolist() == b[0].tolist() and a[1].tolist() == b[1].tolist()


# ------------------------------------------------------------------ merge arithmetic
@pytest.mark.parametrize("seed", range(4))
def test_weighted_merge_conserves_sizes_and_weighted_sum(seed):
    rng = np.random.default_rng(seed)
    n, d = 57, 9
    x = rng.standard_normal((n, d))
    sizes = rng.integers(1, 6, n)
    order_tag = np.arange(n, dtype=np.float64)
    total, wsum = int(sizes.sum()), (sizes[:, None] * x).sum(axis=0)
    for r in (0, 1, 5, 28, 200):
        x2, s2, src, dst, _ = orc.token_merge(x, rng.standard_normal((n, 6)), sizes, r, 1)
        r_eff = orc.removal_count(n, r, 1)
        assert x2.shape == (n - r_eff, d) and s2.shape == (n - r_eff,)
        assert int(s2.sum()) == total and s2.min() >= 1
        assert np.allclose((s2[:, None] * x2).sum(axis=0), wsum, rtol=1e-12, atol=1e-12)
        assert np.array_equal(x2[0], x[0])              # the protected lead token is untouched
        # survivors keep their relative order: un-merged survivors carry their tag unchanged
        t2, _ = orc.merge_apply(order_tag[:, None], np.ones(n, dtype=np.int64), [], [])
        assert np.array_equal(t2[:, 0], order_tag)
        tags, _ = orc.merge_apply(np.where(np.isin(np.arange(n), dst), np.nan, order_tag)[:, None],
                                  sizes, src, dst)
        surv = tags[~np.isnan(tags[:, 0]), 0]
        assert np.all(np.diff(surv) > 0)


def test_merge_apply_hand_example():
    """Three tokens into one, by hand: sizes 2,1,3 and values 1,4,10 -> (2*1+1*4+3*10)/6 = 6."""
    x = np.array([[9.0], [4.0], [1.0], [7.0], [10.0]])
    s = np.array([1, 1, 2, 1, 3])
    x2, s2 = orc.merge_apply(x, s, [2, 4], [1, 1])
    assert x2[:, 0].tolist() == [9.0, 6.0, 7.0] and s2.tolist() == [1, 6, 1]


def test_identity_cases():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((10, 4))
    x2, s2, src, dst, _ = orc.token_merge(x, x, None, 0, 1)
    assert np.array_equal(x2, x) and s2.tolist() == [1] * 10 and src.size == 0
    # size bias with all sizes 1 changes nothing (ln 1 = 0)
    qkv = rng.standard_normal((10, 24))
    assert np.array_equal(orc.attention_heads(qkv, 2), orc.attention_heads(qkv, 2, np.ones(10), True))
    # and with real sizes it equals attention over the token list with every key repeated size times
    sizes = np.array([1, 3, 1, 2, 1, 1, 4, 1, 1, 2])
    rep = np.repeat(np.arange(10), sizes)
    D = 8
    big = qkv[rep]
    ref = orc.attention_heads(big, 2)                   # duplicated keys/values == + ln(size) bias
    got = orc.attention_heads(qkv, 2, sizes, True)
    first = np.concatenate([[0], np.cumsum(sizes)[:-1]])
    assert np.allclose(got, ref[first], atol=1e-12)
    assert D == qkv.shape[1] // 3


# ------------------------------------------------------------------ whole encoder with adaptation
def test_encoder_invariants_on_tiny_config():
    cfg = synth.config("tiny")
    layers = synth.all_weights(cfg)
    toks, prm, P, R = synth.batch(cfg)
    outs = []
    for q in range(cfg.B):
        x0, _ = orc.prompt_prepend(toks[q], prm[q], cfg.n_lead)
        o = orc.encoder_forward_query(x0, layers, R[q], H=cfg.H, ln_eps=cfg.ln_eps, n_lead=cfg.n_lead)
        outs.append(o)
        assert o["lengths"] == orc.length_schedule(cfg.n0, P[q], R[q], cfg.n_lead, cfg.L) == [201, 193, 185]
        assert int(o["sizes"].sum()) == cfg.n0 + P[q] and o["sizes"].min() >= 1
        for (src, dst), n in zip(o["trace"], o["lengths"]):
            orc.validate_decision(n, 8, 1, src, dst)
        assert o["sizes"][0] == 1                       # class token never merged
        assert min(m["rank_margin"] for m in o["margins"]) > 1e-6
        assert min(m["argmax_margin"] for m in o["margins"]) > 1e-6
    # query independence: the batch routine is the per-query routine
    x0s = [orc.prompt_prepend(t, p, 1)[0] for t, p in zip(toks, prm)]
    both = orc.encoder_forward(x0s, layers, R, H=cfg.H, ln_eps=cfg.ln_eps, n_lead=1)
    for a, b in zip(outs, both):
        assert np.array_equal(a["x"], b["x"])


def test_lockstep_adoption_counts_disagreements_and_applies_given_decision():
    rng = np.random.default_rng(9)
    D, H, F, n = 16, 2, 32, 21
    layers = _rand_layers(rng, 2, D, F)
    x0 = rng.standard_normal((n, D))
    own = orc.encoder_forward_query(x0, layers, 3, H=H, ln_eps=1e-6, n_lead=1)
    same = orc.encoder_forward_query(x0, layers, 3, H=H, ln_eps=1e-6, n_lead=1, adopt=own["trace"])
    assert same["disagree"] == [0, 0] and np.array_equal(same["x"], own["x"])
    src, dst = own["trace"][0]
    other_a = next(a for a in range(2, n, 2) if a not in set(src.tolist()))
    forced = [(np.concatenate([src[:-1], [other_a]]), np.concatenate([dst[:-1], [1]])), None]
    first = orc.encoder_forward_query(x0, layers[:1], 3, H=H, ln_eps=1e-6, n_lead=1, adopt=forced[:1])
    assert first["disagree"] == [1]
    assert not np.array_equal(first["x"], orc.encoder_forward_query(x0, layers[:1], 3, H=H, ln_eps=1e-6, n_lead=1)["x"])
    with pytest.raises(ValueError):
        orc.validate_decision(n, 3, 1, [0, 2, 4], [1, 1, 1])      # protected token as a source
    with pytest.raises(ValueError):
        orc.validate_decision(n, 3, 1, [2, 2, 4], [1, 1, 1])      # a token merged twice


def test_storage_modes_round_where_stated():
    rng = np.random.default_rng(10)
    D, H, F, n = 32, 2, 64, 15
    layers = [{k: synth.round_to_bf16(v.astype(np.float32)) for k, v in w.items()} for w in _rand_layers(rng, 2, D, F, 0.1)]
    x0 = synth.round_to_bf16(rng.standard_normal((n, D)).astype(np.float32))
    f64 = orc.encoder_forward_query(x0, layers, 2, H=H, ln_eps=1e-6, n_lead=1)
    b16 = orc.encoder_forward_query(x0, layers, 2, H=H, ln_eps=1e-6, n_lead=1, storage="bf16")
    assert np.array_equal(b16["x"], orc.round_storage(b16["x"], "f32"))      # the residual stream is float32
    assert not np.array_equal(b16["x"], orc.round_storage(b16["x"], "bf16"))
    err = np.max(np.abs(b16["x"] - f64["x"])) / np.max(np.abs(f64["x"]))
    assert 0 < err < 3e-2
    f32 = orc.encoder_forward_query(x0, layers, 2, H=H, ln_eps=1e-6, n_lead=1, storage="f32")
    assert np.max(np.abs(f32["x"] - f64["x"])) / np.max(np.abs(f64["x"])) < 1e-5


# ------------------------------------------------------------------ planted mistakes are caught
def test_pins_catch_planted_mistakes(monkeypatch):
    """Mutate the oracle on the CPU and check that a pin notices: guards against vacuous pins."""
    rng = np.random.default_rng(12)
    m = rng.standard_normal((12, 5))
    want = _brute_force_edges(m, 4, 1)
    # (a) swapped sets (odd -> A)
    bad = orc.merge_plan(m[::-1].copy(), 4, 1)
    assert list(zip(bad[0].tolist(), bad[1].tolist())) != want
    # (b) unweighted average breaks the conserved weighted sum
    x = rng.standard_normal((9, 3)); s = np.array([1, 2, 3, 1, 1, 2, 1, 1, 5])
    x2, s2 = orc.merge_apply(x, s, [2, 6], [3, 3])
    assert np.allclose((s2[:, None] * x2).sum(0), (s[:, None] * x).sum(0))
    naive = (x[3] + x[2] + x[6]) / 3
    assert not np.allclose(naive, x2[2])
    # (c) missing 1/sqrt(d_k): the library SDPA comparison would fail
    monkeypatch.setattr(orc.math, "sqrt", lambda v: 1.0)
    qkv = rng.standard_normal((7, 3 * 8))
    t = torch.from_numpy(qkv)
    q, k, v = (t[:, i * 8:(i + 1) * 8].reshape(7, 2, 4).transpose(0, 1) for i in range(3))
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v).transpose(0, 1).reshape(7, 8).numpy()
    assert not np.allclose(orc.attention_heads(qkv, 2), ref, atol=1e-6)


def test_per_layer_prompting_pins_catch_planted_mistakes(monkeypatch):
    """A prompting step that writes one row too late, or appends instead of inserting, must break the
    closed form of the residual-free model."""
    rng = np.random.default_rng(13)
    n0, P, D, H, F, L = 6, 2, 8, 2, 16, 3
    layers = _rand_layers(rng, L, D, F)
    off = [dict(w, w_proj=np.zeros((D, D)), b_proj=np.zeros(D), w_fc2=np.zeros((D, F)), b_fc2=np.zeros(D)) for w in layers]
    toks = rng.standard_normal((n0, D))
    prm = [rng.standard_normal((P, D)) for _ in range(L)]
    x0, _ = orc.prompt_prepend(toks, prm[0], 1)
    want_rep = np.concatenate([toks[:1], prm[L - 1], toks[1:]])
    want_grw = np.concatenate([toks[:1]] + [prm[l] for l in range(L - 1, -1, -1)] + [toks[1:]])
    good = orc.deep_prompt_step

    def late(x, sizes, prompts, n_lead, mode):
        return good(x, sizes, prompts, n_lead + 1, mode)

    def appended(x, sizes, prompts, n_lead, mode):
        if mode == "grow":
            return np.concatenate([x, prompts]), np.concatenate([sizes, np.ones(len(prompts), dtype=sizes.dtype)])
        return good(x, sizes, prompts, n_lead, mode)

    monkeypatch.setattr(orc, "deep_prompt_step", late)
    bad = orc.encoder_forward_query(x0, off, 0, H=H, ln_eps=1e-6, n_lead=1, deep_prompts=prm, deep_mode="replace")
    assert not np.array_equal(bad["x"], want_rep)
    monkeypatch.setattr(orc, "deep_prompt_step", appended)
    bad = orc.encoder_forward_query(x0, off, 0, H=H, ln_eps=1e-6, n_lead=1, deep_prompts=prm, deep_mode="grow")
    assert not np.array_equal(bad["x"], want_grw)


# ------------------------------------------------------------------ model ends (R14)
@pytest.mark.parametrize("with_cls", [True, False])
def test_patch_embed_matches_library_convolution(with_cls):
    """Splitting into p x p patches and projecting linearly is a convolution with kernel = stride = p
    (torch.nn.functional.conv2d, float64); class token and position embedding placed by hand."""
    rng = np.random.default_rng(21)
    C, Hi, Wi, p, D = 3, 8, 12, 4, 10
    img = rng.standard_normal((C, Hi, Wi))
    w = rng.standard_normal((D, C, p, p))
    b = rng.standard_normal(D)
    cls = rng.standard_normal(D) if with_cls else None
    N = (Hi // p) * (Wi // p)
    pos = rng.standard_normal((N + (1 if with_cls else 0), D))
    got = orc.patch_embed(img, w, b, cls, pos, p)
    conv = torch.nn.functional.conv2d(torch.from_numpy(img)[None], torch.from_numpy(w), torch.from_numpy(b), stride=p)
    ref = conv[0].flatten(1).T.numpy()          # [N, D], patches row by row
    if with_cls:
        ref = np.concatenate([cls[None], ref], axis=0)
    ref = ref + pos
    assert got.shape == ref.shape
    assert np.max(np.abs(got - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))
    # a planted mistake (patches walked column by column) is caught on a non-square patch grid
    wrong = orc.patch_embed(img.transpose(0, 2, 1), w.transpose(0, 1, 3, 2), b, cls, pos, p)
    assert not np.allclose(wrong, ref)
    with pytest.raises(ValueError):
        orc.patch_embed(img[:, :7], w, b, cls, pos, p)


def test_task_head_matches_library_norm_and_linear():
    rng = np.random.default_rng(22)
    n, D, K = 6, 12, 5
    x = rng.standard_normal((n, D))
    g, bb = 1 + 0.1 * rng.standard_normal(D), 0.1 * rng.standard_normal(D)
    w, b = rng.standard_normal((K, D)), rng.standard_normal(K)
    got = orc.task_head(x, g, bb, w, b, 1e-6)
    t = torch.nn.functional.layer_norm(torch.from_numpy(x[0]), (D,), torch.from_numpy(g), torch.from_numpy(bb), 1e-6)
    ref = torch.nn.functional.linear(t, torch.from_numpy(w), torch.from_numpy(b)).numpy()
    assert got.shape == (K,)
    assert np.max(np.abs(got - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))
    # only the first token counts
    x2 = x.copy(); x2[1:] += 1.0
    assert np.array_equal(orc.task_head(x2, g, bb, w, b, 1e-6), got)


# ------------------------------------------------------------------ merge metric and where the merge sits
def _independent_adapted_encoder(x0, layers, r, D, H, F, n_lead, eps=1e-6, metric_from="K",
                                 head_layout="H_dh", keys_of="this_layer", merge_at="after_attention_residual"):
    """Sec. III-B stated independently of the oracle: per block, torch's own pre-norm pieces
    (norm1, self_attn, out_proj residual, norm2, linear1, GELU, linear2 residual), the metric from
    torch layer_norm + linear with ONLY the key rows D..2D of w_qkv, the head mean written as explicit
    Python loops, edges by the brute-force enumeration, the weighted average by explicit loops over
    rows, and the merge between the attention residual and the MLP.  The keyword arguments switch in
    the plausible misreadings (metric from Q or V, heads and head width swapped, the previous layer's
    keys, merging at another point of the block) so that a test can show they give other results.
    (Merging the stream and the attention branch separately and adding them afterwards is NOT another
    result: the size-weighted average is linear, so it equals merging their sum; the placements that
    can be told apart are in front of the attention and behind the MLP.)"""
    F_ = torch.nn.functional
    dh = D // H
    x = torch.from_numpy(np.asarray(x0, dtype=np.float64))
    sizes = [1] * x.shape[0]
    traces = []
    prev_metric = None

    def plan(metric_rows, n_now):
        r_eff = max(0, min(r, (n_now - n_lead) // 2))
        return _brute_force_edges(np.asarray(metric_rows, dtype=np.float64)[:n_now], r_eff, n_lead)

    def apply(x, sizes, edges):
        n_now = x.shape[0]
        rows = [x[i].clone() for i in range(n_now)]
        new_sizes = list(sizes)
        for b in sorted({b for _, b in edges}):
            tot = sizes[b]
            acc = sizes[b] * x[b]
            for a in sorted(a for a, bb in edges if bb == b):
                acc = acc + sizes[a] * x[a]
                tot += sizes[a]
            rows[b] = acc / tot
            new_sizes[b] = tot
        gone = {a for a, _ in edges}
        keep = [i for i in range(n_now) if i not in gone]
        return torch.stack([rows[i] for i in keep]), [new_sizes[i] for i in keep]

    with torch.no_grad():
        for m, w in zip(_torch_encoder(layers, D, H, F, eps), layers):
            n_now = x.shape[0]
            h = F_.layer_norm(x, (D,), torch.from_numpy(w["ln1_g"]), torch.from_numpy(w["ln1_b"]), eps)
            third = {"Q": 0, "K": 1, "V": 2}[metric_from]
            wk = torch.from_numpy(np.asarray(w["w_qkv"], dtype=np.float64))[third * D:(third + 1) * D]
            bk = torch.from_numpy(np.asarray(w["b_qkv"], dtype=np.float64))[third * D:(third + 1) * D]
            keys = F_.linear(h, wk, bk).numpy()                        # [n, D], heads side by side
            metric = [[0.0] * dh for _ in range(n_now)]
            for i in range(n_now):
                for hd in range(H):
                    for j in range(dh):
                        col = hd * dh + j if head_layout == "H_dh" else j * H + hd
                        metric[i][j] += keys[i][col] / H
            use = metric if (keys_of == "this_layer" or prev_metric is None) else prev_metric
            prev_metric = metric
            if merge_at == "before_attention":
                edges = plan(use, n_now)
                x, sizes = apply(x, sizes, edges)
                traces.append(edges)
                x = x + m.self_attn(m.norm1(x)[None], m.norm1(x)[None], m.norm1(x)[None], need_weights=False)[0][0]
            else:
                attn = m.self_attn(m.norm1(x)[None], m.norm1(x)[None], m.norm1(x)[None], need_weights=False)[0][0]
                x = x + attn
                if merge_at == "after_attention_residual":
                    edges = plan(use, n_now)
                    x, sizes = apply(x, sizes, edges)
                    traces.append(edges)
            x = x + m.linear2(F_.gelu(m.linear1(m.norm2(x))))
            if merge_at == "after_mlp":
                edges = plan(use, n_now)
                x, sizes = apply(x, sizes, edges)
                traces.append(edges)
    return x.numpy(), sizes, traces


@pytest.mark.parametrize("L,n,r,n_lead", [(1, 13, 3, 1), (2, 17, 4, 1), (2, 12, 5, 0), (3, 21, 2, 1)])
def test_merge_metric_and_placement_against_independent_blocks(L, n, r, n_lead):
    """Sec. III-B: the similarity comes from the layer's own multi-head attention (head-averaged keys,
    R3) and the merging module sits between the attention residual and the MLP.  The oracle's trace,
    sizes and output must equal the independent statement above; every misreading must not."""
    rng = np.random.default_rng(100 + L * 7 + n)
    D, H, F = 24, 4, 40                                  # d_h = 6 != H, so a swapped reshape shows
    layers = _rand_layers(rng, L, D, F, scale=0.35)
    x0 = rng.standard_normal((n, D))
    got = orc.encoder_forward_query(x0, layers, r, H=H, ln_eps=1e-6, n_lead=n_lead)
    ref_x, ref_s, ref_tr = _independent_adapted_encoder(x0, layers, r, D, H, F, n_lead)
    assert [list(zip(s.tolist(), d.tolist())) for s, d in got["trace"]] == ref_tr
    assert got["sizes"].tolist() == ref_s
    assert got["x"].shape == ref_x.shape
    assert np.max(np.abs(got["x"] - ref_x)) <= 1e-11 * max(1.0, np.max(np.abs(ref_x)))
    assert any(len(t) for t in ref_tr)
    # the misreadings give something else, so an oracle that had taken one would fail the lines above
    wrong = [dict(metric_from="Q"), dict(metric_from="V"), dict(head_layout="dh_H"),
             dict(merge_at="before_attention"), dict(merge_at="after_mlp")]
    if L > 1:
        wrong += [dict(keys_of="previous_layer")]
    for kw in wrong:
        bad_x, bad_s, bad_tr = _independent_adapted_encoder(x0, layers, r, D, H, F, n_lead, **kw)
        same_trace = [list(zip(s.tolist(), d.tolist())) for s, d in got["trace"]] == bad_tr
        same_x = bad_x.shape == got["x"].shape and np.max(np.abs(got["x"] - bad_x)) <= 1e-9
        assert not (same_trace and same_x), kw


def test_merge_metric_hand_example():
    """Two heads of width three: the key third of a row is [1 2 3 | 4 5 6], its head mean is
    (2.5, 3.5, 4.5) by hand.  Taking the Q or V third, or reading the row as three heads of two, gives
    other numbers."""
    row = np.array([[10., 20., 30., 40., 50., 60., 1., 2., 3., 4., 5., 6., -1., -2., -3., -4., -5., -6.],
                    [0., 0., 0., 0., 0., 0., 2., 0., -2., 4., 2., 0., 9., 9., 9., 9., 9., 9.]])
    m = orc.merge_metric_from_keys(row, 2)
    assert m.shape == (2, 3)
    assert m.tolist() == [[2.5, 3.5, 4.5], [3.0, 1.0, -1.0]]


def test_pins_catch_planted_metric_mistakes(monkeypatch):
    """Plant the slips in the oracle itself and check the independent-block pin notices each one."""
    rng = np.random.default_rng(31)
    L, n, r, D, H, F = 2, 15, 3, 24, 4, 40
    layers = _rand_layers(rng, L, D, F, scale=0.35)
    x0 = rng.standard_normal((n, D))
    ref_x, ref_s, ref_tr = _independent_adapted_encoder(x0, layers, r, D, H, F, 1)

    def oracle_agrees():
        try:
            got = orc.encoder_forward_query(x0, layers, r, H=H, ln_eps=1e-6, n_lead=1)
        except Exception:
            return False
        return ([list(zip(s.tolist(), d.tolist())) for s, d in got["trace"]] == ref_tr
                and got["x"].shape == ref_x.shape and np.max(np.abs(got["x"] - ref_x)) <= 1e-9)

    assert oracle_agrees()
    dh = D // H
    state = {}

    def from_q(qkv, H_):
        return qkv[:, 0:D].reshape(qkv.shape[0], H_, dh).mean(axis=1)

    def from_v(qkv, H_):
        return qkv[:, 2 * D:3 * D].reshape(qkv.shape[0], H_, dh).mean(axis=1)

    def swapped(qkv, H_):
        return qkv[:, D:2 * D].reshape(qkv.shape[0], dh, H_).mean(axis=2)

    def no_head_mean(qkv, H_):
        return qkv[:, D:D + dh]                          # first head only

    good = orc.merge_metric_from_keys

    def previous_layer(qkv, H_):
        now = good(qkv, H_)
        old = state.get("m")
        state["m"] = now
        return now if old is None else old[:now.shape[0]]

    for slip in (from_q, from_v, swapped, no_head_mean, previous_layer):
        state.clear()
        monkeypatch.setattr(orc, "merge_metric_from_keys", slip)
        assert not oracle_agrees(), slip.__name__
    monkeypatch.setattr(orc, "merge_metric_from_keys", good)
    assert oracle_agrees()


def test_edge_deficit_hand_example():
    """Six unit vectors from 3-4-5 triangles, so every cosine is a short decimal.  A = positions 0, 2, 4
    = (0.8, 0.6), (0.6, 0.8), (-0.6, 0.8); B = positions 1, 3, 5 = (1, 0), (0, 1), (0.6, 0.8).
    Similarities by hand:      b=1    b=3    b=5
                        a=0    0.8    0.6    0.96
                        a=2    0.6    0.8    1.0
                        a=4   -0.6    0.8    0.28
    best = (0.96, 1.0, 0.8); with two edges kept the second best edge has 0.96.  The deficit of an
    edge (a, b) is how much its similarity falls short of a's best and of the last kept edge."""
    m = np.array([[0.8, 0.6], [1.0, 0.0], [0.6, 0.8], [0.0, 1.0], [-0.6, 0.8], [0.6, 0.8]])
    src, dst, info = orc.merge_plan(m, 2, 0)
    assert list(zip(src.tolist(), dst.tolist())) == [(2, 5), (0, 5)]
    assert np.allclose(info["sim"], [[0.8, 0.6, 0.96], [0.6, 0.8, 1.0], [-0.6, 0.8, 0.28]], atol=1e-15)
    assert np.allclose(info["best"], [0.96, 1.0, 0.8], atol=1e-15) and abs(info["kth"] - 0.96) < 1e-15
    assert abs(info["rank_margin"] - 0.16) < 1e-12 and abs(info["argmax_margin"] - 0.16) < 1e-12
    want = {(2, 5): 0.0, (0, 5): 0.0, (4, 3): 0.16, (0, 1): 0.16, (2, 1): 0.4, (4, 5): 0.68,
            (4, 1): 1.56, (0, 3): 0.36, (2, 3): 0.2}
    for (a, b), d in want.items():
        assert abs(orc.edge_deficit(info, a, b) - d) < 1e-12, (a, b)
    # with a protected lead token row 0 cannot merge: the kept edges become (2,5) and (4,3), kth = 0.8
    src, dst, info = orc.merge_plan(m, 2, 1)
    assert list(zip(src.tolist(), dst.tolist())) == [(2, 5), (4, 3)]
    assert abs(orc.edge_deficit(info, 4, 1) - 1.4) < 1e-12 and orc.edge_deficit(info, 4, 3) == 0.0


def test_float32_arithmetic_mode_follows_the_float64_oracle():
    """The benchmark's second CPU figure runs the oracle's steps in float32 arithmetic: without merging
    it must agree with the float64 oracle to float32 accuracy, and with merging it must obey the same
    shape law and size conservation."""
    rng = np.random.default_rng(41)
    D, H, F, n, L = 32, 4, 64, 19, 3
    layers = _rand_layers(rng, L, D, F, 0.2)
    x0 = rng.standard_normal((n, D))
    a = orc.encoder_forward_query(x0, layers, 0, H=H, ln_eps=1e-6, n_lead=1)
    b = orc.encoder_forward_query(x0, layers, 0, H=H, ln_eps=1e-6, n_lead=1, arith="f32")
    assert np.max(np.abs(a["x"] - b["x"])) / np.max(np.abs(a["x"])) < 1e-5
    c = orc.encoder_forward_query(x0, layers, 3, H=H, ln_eps=1e-6, n_lead=1, arith="f32")
    assert c["lengths"] == orc.length_schedule(n, 0, 3, 1, L) and int(c["sizes"].sum()) == n
    d = orc.encoder_forward_query(x0, layers, 3, H=H, ln_eps=1e-6, n_lead=1)
    if all(np.array_equal(s1, s2) and np.array_equal(d1, d2) for (s1, d1), (s2, d2) in zip(c["trace"], d["trace"])):
        assert np.max(np.abs(c["x"] - d["x"])) / np.max(np.abs(d["x"])) < 1e-4
    with pytest.raises(ValueError):
        orc.encoder_forward_query(x0, layers, 0, H=H, ln_eps=1e-6, n_lead=1, arith="f16")
