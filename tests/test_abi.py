"""CPU-side checks of the C-ABI library: it loads without a GPU, exports every symbol the header
declares, and its pure-host functions agree with the oracle's closed forms."""
import ctypes
import os
import re

import pytest

import paper_2401_05031_amd as otas
from paper_2401_05031_amd import binding
from oracle import otas_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _ensure_built():
    if not os.path.exists(otas.lib_path()):
        from paper_2401_05031_amd import build
        build.build(verbose=False)


def test_library_exports_every_declared_symbol():
    _ensure_built()
    header = "".join(open(os.path.join(ROOT, "include", f)).read()
                     for f in sorted(os.listdir(os.path.join(ROOT, "include"))) if f.endswith(".h"))
    declared = set(re.findall(r"\b(otas_[a-z_0-9]+)\s*\(", header))
    declared -= {"otas_ctx", "otas_sched"}
    assert declared == set(binding.EXPORTED)
    lib = ctypes.CDLL(otas.lib_path())
    for name in declared:
        assert hasattr(lib, name), name


def test_schedule_matches_oracle_closed_form():
    _ensure_built()
    for n0, P, r, nl, L in [(197, 4, 8, 1, 2), (197, 0, 16, 1, 12), (197, 0, 24, 1, 24), (257, 10, 12, 1, 32),
                            (8, 0, 100, 0, 5), (1, 0, 3, 1, 4), (2, 0, 0, 0, 3)]:
        assert otas.otas_schedule(n0, P, r, nl, L) == orc.length_schedule(n0, P, r, nl, L)


def test_host_side_argument_errors():
    _ensure_built()
    with pytest.raises(otas.OtasError) as e:
        otas.otas_schedule(5, 0, -1, 1, 2)
    assert e.value.status == 1
    with pytest.raises(otas.OtasError):
        otas.otas_schedule(0, 0, 1, 1, 2)          # shorter than the protected lead
    assert otas.otas_strerror(0) == "ok" and "workspace" in otas.otas_strerror(3)
    lib = otas.load_library()
    assert lib.otas_merge_workspace_bytes(0, 10) == 0 and lib.otas_merge_workspace_bytes(2, 10) > 0
    assert lib.otas_workspace_bytes(None, 1, 1) == 0
    # NULL context / pointers are rejected before anything touches a device
    assert lib.otas_encoder_forward(None, None, None, None, 1, 0, None, 0, None, None, None, None, None) == 1
    assert lib.otas_token_merge(None, None, None, 64, None, None, None, 1, None, 0, None, None, None, None, None) == 1
    assert lib.otas_prompt_prepend(None, None, None, None, None, 1, None, None) == 1
    assert lib.otas_prompt_prepend_pool(None, None, None, None, 0, None, None, 1, None, None) == 1
    assert lib.otas_token_merge_static(None, None, None, 64, None, None, None, 1, None, None, None, None, None) == 1
    assert lib.otas_linear_kernel(None, 2, None, None, None, None, 1, 8, 64, 0, None) == 1
    assert lib.otas_linear_choice(None, 128, 768, 768, 0) == -1
    assert lib.otas_clock_probe_start(None, 16) == 1
    assert lib.otas_clock_probe_read(None, None, 0, None) == 1
    assert lib.otas_create(None, None, None, None) == 1


def test_rate_table_host_function_rejects_bad_input():
    _ensure_built()
    import numpy as np
    with pytest.raises(otas.OtasError):
        otas.otas_sched_rate_table([0, -5], np.array([[1e-3, -1e-3]]))       # a non-positive latency
    with pytest.raises(ValueError):
        otas.otas_sched_rate_table([0, -5], np.array([[1e-3]]))              # wrong table shape
    assert otas.otas_sched_rate_table([0], np.array([[1e-3]])) == []         # one gamma: it is the overflow row
