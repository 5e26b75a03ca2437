"""CPU calibration of what "near-tie" means for end-to-end bf16 runs.

The oracle, with bf16 storage rounding, is run twice on the ViT-B r=16 workload: once as is and
once with ONE input element moved by one bf16 unit.  The two trajectories decorrelate to the bf16
noise floor (a difference d ahead of a rounding with unit u is ~sqrt(d*u) behind it), so a small
share of merge decisions flips although both runs are "the oracle".  Any independent bf16
implementation -- the HIP path included -- can only be expected to agree with the oracle to this
degree end to end; the GPU tests therefore apply the 0.1 % bar on decisions where both sides see
identical inputs (block by block), and end to end they require every differing edge to be within
NEAR_TIE of the oracle's own choice.  This test pins NEAR_TIE to the measured floor."""
import numpy as np

import otas_synth as synth
from oracle import otas_oracle as orc

NEAR_TIE = 4e-3   # measured: CPU self-disagreement 0.8e-3, GPU end to end <= 1.7e-3


def test_one_ulp_input_change_moves_decisions_only_at_near_ties():
    cfg = synth.config("vitb_r16")
    layers = synth.all_weights(cfg)
    dec = dis = 0
    deficits, errs = [], []
    for q in (0, 1):
        x0 = synth.query_tokens(cfg, q).astype(np.float64)
        a = orc.encoder_forward_query(x0, layers, 16, H=cfg.H, ln_eps=cfg.ln_eps, n_lead=1, storage="bf16")
        x1 = x0.copy()
        bits = np.float32(x0[5, 7]).view(np.uint32) + np.uint32(0x10000)   # one bf16 unit in the last place
        x1[5, 7] = float(bits.view(np.float32))
        assert x1[5, 7] != x0[5, 7] and orc.round_storage(x1, "bf16")[5, 7] == x1[5, 7]
        b = orc.encoder_forward_query(x1, layers, 16, H=cfg.H, ln_eps=cfg.ln_eps, n_lead=1, storage="bf16",
                                      adopt=a["trace"])
        dec += sum(s.size for s, _ in a["trace"])
        dis += sum(b["disagree"])
        deficits += b["deficits"]
        errs.append(np.max(np.abs(a["x"] - b["x"])) / np.max(np.abs(a["x"])))
    print("decisions", dec, "flipped", dis, "max deficit", max(deficits, default=0.0), "rel diff", errs)
    assert dec == 2 * (16 * 11 + 10)
    assert max(errs) > 1e-3                  # the trajectories really did decorrelate ...
    assert max(errs) < 2e-2                  # ... to the bf16 noise floor, not beyond
    assert max(deficits, default=0.0) <= NEAR_TIE
    assert dis <= 0.015 * dec
