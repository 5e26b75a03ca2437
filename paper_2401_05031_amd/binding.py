"""ctypes binding of libotas.so.

The functions mirror the C ABI one to one (same names, same argument order) and only marshal
arguments: torch tensors become device pointers, Python lists become host int32 arrays.  There is
no fallback: if the library is missing or fails to load, importing a symbol raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

OTAS_F32, OTAS_BF16 = 0, 1
OTAS_FLAG_SIZE_BIAS, OTAS_FLAG_TRACE = 1, 2
OTAS_PROMPT_REPLACE, OTAS_PROMPT_GROW = 1, 2
OTAS_STATIC_MERGE_MAX_ROWS, OTAS_STATIC_MERGE_MAX_QUERIES = 65536, 1024
OTAS_LINEAR_KERNELS = 8
OTAS_CLOCK_PROBE_MAX_SAMPLES = 65536
_WEIGHT_FIELDS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_proj", "b_proj",
                  "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


class OtasError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {otas_strerror(status)} (status {status})")


class _TaskHead(C.Structure):
    _fields_ = [("w", C.c_void_p), ("b", C.c_void_p), ("classes", C.c_int32)]


class _ModelDesc(C.Structure):
    _fields_ = [("L", C.c_int32), ("D", C.c_int32), ("H", C.c_int32), ("F", C.c_int32),
                ("dtype", C.c_int32), ("ln_eps", C.c_float), ("n_lead", C.c_int32)]


class _LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _WEIGHT_FIELDS]


class _SchedParams(C.Structure):
    _fields_ = [("delta", C.c_double), ("eta", C.c_double), ("mu", C.c_double), ("kappa", C.c_double),
                ("epsilon", C.c_int32), ("beta", C.c_int32)]


OTAS_GAMMA_SKIP, OTAS_GAMMA_UNDECIDED = -1, -2
_I32P = C.POINTER(C.c_int32)
_I64P = C.POINTER(C.c_int64)
_F64P = C.POINTER(C.c_double)
_LIB = None


def lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libotas.so")


def load_library():
    """Load libotas.so (built in-tree by paper_2401_05031_amd/build.py).  Raises if absent."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is not built: run `python -m paper_2401_05031_amd.build` "
                          "(there is no CPU fallback)")
    # torch ships its own copy of the HIP runtime under the same soname as the system one; load
    # torch first so that the library, torch's allocator and torch's streams share ONE runtime.
    import torch  # noqa: F401
    lib = C.CDLL(path)
    vp, i32, i64, u32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_size_t
    sigs = {
        "otas_create": (i32, [C.POINTER(vp), C.POINTER(_ModelDesc), C.POINTER(_LayerWeights), vp]),
        "otas_destroy": (i32, [vp]),
        "otas_schedule": (i32, [i32, i32, i32, i32, i32, _I32P]),
        "otas_workspace_bytes": (sz, [vp, i32, i64]),
        "otas_merge_workspace_bytes": (sz, [i32, i64]),
        "otas_prompt_prepend": (i32, [vp, vp, _I32P, vp, _I32P, i32, vp, _I32P]),
        "otas_prompt_prepend_pool": (i32, [vp, vp, _I32P, vp, i64, _I32P, _I32P, i32, vp, _I32P]),
        "otas_token_merge": (i32, [vp, vp, vp, i32, vp, _I32P, _I32P, i32, vp, sz, vp, vp, _I32P, vp, vp]),
        "otas_token_merge_static": (i32, [vp, vp, vp, i32, vp, _I32P, _I32P, i32, vp, vp, _I32P, vp, vp]),
        "otas_encoder_forward": (i32, [vp, vp, _I32P, _I32P, i32, u32, vp, sz, vp, vp, _I32P, vp, vp]),
        "otas_encoder_layers": (i32, [vp, i32, i32, vp, vp, _I32P, _I32P, i32, u32, vp, sz, vp, vp, _I32P, vp, vp]),
        "otas_encoder_forward_deep": (i32, [vp, vp, _I32P, i32, i32, vp, _I32P, vp, sz, vp, vp, _I32P]),
        "otas_patch_embed_workspace_bytes": (sz, [vp, i32, i32, i32, i32, i32]),
        "otas_patch_embed": (i32, [vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp, _I32P]),
        "otas_task_heads": (i32, [vp, vp, _I32P, _I32P, i32, C.POINTER(_TaskHead), i32, vp, vp, vp, i32]),
        "otas_layer_norm": (i32, [vp, vp, vp, vp, i64, vp]),
        "otas_linear": (i32, [vp, vp, vp, vp, vp, i64, i32, i32, i32, vp]),
        "otas_attention": (i32, [vp, vp, vp, _I32P, i32, u32, vp]),
        "otas_linear_choice": (i32, [vp, i64, i32, i32, i32]),
        "otas_linear_kernel": (i32, [vp, i32, vp, vp, vp, vp, i64, i32, i32, i32, vp]),
        "otas_strerror": (C.c_char_p, [i32]),
        "otas_timing_enable": (i32, [vp, i32]),
        "otas_timing_kinds": (i32, []),
        "otas_timing_kind_name": (C.c_char_p, [i32]),
        "otas_timing_read": (i32, [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
        "otas_timing_read_launches": (i32, [vp, i32, _I32P, C.POINTER(C.c_float)]),
        "otas_timing_overhead_ms": (C.c_float, [vp]),
        "otas_set_lanes": (i32, [vp, i32]),
        "otas_clock_probe_start": (i32, [vp, i32]),
        "otas_clock_probe_read": (i32, [vp, C.POINTER(C.c_float), i32, _I32P]),
        "otas_splitk_factor": (i32, [vp, C.c_int64, i32, i32, i32]),
        "otas_splitk_room": (i32, [vp, C.c_int64, C.c_int64]),
        "otas_sched_create": (i32, [C.POINTER(_SchedParams), i32, _I32P, i32, _F64P, _F64P, i32, _F64P, _I32P,
                                    C.POINTER(vp)]),
        "otas_sched_destroy": (None, [vp]),
        "otas_sched_rate_table": (i32, [i32, _I32P, i32, _F64P, _F64P, _I32P, _I32P]),
        "otas_sched_add_query": (i32, [vp, i64, C.c_double, C.c_double, C.c_double, i32, _I32P]),
        "otas_sched_allocate": (i32, [vp, C.c_double, C.c_double, i32, _F64P]),
        "otas_sched_num_batches": (i32, [vp]),
        "otas_sched_batch_info": (i32, [vp, i32, _I32P, _F64P, _F64P, _F64P, _I32P]),
        "otas_sched_batch_queries": (i32, [vp, i32, _I64P, _I32P, i32, _I32P]),
        "otas_sched_estimate": (i32, [vp, i32, i32, _F64P, _F64P]),
        "otas_sched_remove": (i32, [vp, i32]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)          # AttributeError if a declared symbol is not exported
        fn.restype, fn.argtypes = res, args
    _LIB = lib
    return lib


EXPORTED = ("otas_create", "otas_destroy", "otas_schedule", "otas_workspace_bytes",
            "otas_merge_workspace_bytes", "otas_prompt_prepend", "otas_prompt_prepend_pool", "otas_token_merge", "otas_token_merge_static",
            "otas_encoder_forward", "otas_encoder_layers", "otas_encoder_forward_deep", "otas_patch_embed_workspace_bytes", "otas_patch_embed", "otas_task_heads", "otas_layer_norm", "otas_linear", "otas_attention", "otas_linear_kernel", "otas_linear_choice", "otas_strerror",
            "otas_timing_enable", "otas_timing_kinds", "otas_timing_kind_name", "otas_timing_read",
            "otas_timing_read_launches", "otas_timing_overhead_ms", "otas_set_lanes", "otas_splitk_factor", "otas_splitk_room",
            "otas_clock_probe_start", "otas_clock_probe_read",
            "otas_sched_create", "otas_sched_destroy", "otas_sched_rate_table", "otas_sched_add_query", "otas_sched_allocate",
            "otas_sched_num_batches", "otas_sched_batch_info", "otas_sched_batch_queries", "otas_sched_estimate",
            "otas_sched_remove")


def otas_strerror(status: int) -> str:
    return load_library().otas_strerror(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise OtasError(status, where)


def _i32(values: Sequence[int]):
    a = np.ascontiguousarray(np.asarray(values, dtype=np.int32))
    return a, a.ctypes.data_as(_I32P)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def otas_schedule(n0: int, P: int, r: int, n_lead: int, L: int) -> List[int]:
    out = (C.c_int32 * (L + 1))()
    _check(load_library().otas_schedule(n0, P, r, n_lead, L, out), "otas_schedule")
    return list(out)


class Context:
    """Owns an otas_ctx.  Methods carry the C entry points' names and argument meaning; tensors
    must be contiguous torch tensors on the GPU, of the model's dtype unless noted."""

    def __init__(self, L: int, D: int, H: int, F: int, dtype: int, ln_eps: float, n_lead: int,
                 layers: Sequence[dict], stream: Optional[int] = None):
        import torch
        self._lib = load_library()
        self.L, self.D, self.H, self.F, self.dtype, self.n_lead = L, D, H, F, dtype, n_lead
        self.torch_dtype = torch.float32 if dtype == OTAS_F32 else torch.bfloat16
        self._keep = [dict(w) for w in layers]           # the library keeps pointers, not copies
        arr = (_LayerWeights * L)()
        for l, w in enumerate(self._keep):
            for f in _WEIGHT_FIELDS:
                t = w[f]
                assert t.is_cuda and t.is_contiguous() and t.dtype == self.torch_dtype, f
                setattr(arr[l], f, t.data_ptr())
        desc = _ModelDesc(L, D, H, F, dtype, ln_eps, n_lead)
        self._h = C.c_void_p()
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        self.stream = stream
        _check(self._lib.otas_create(C.byref(self._h), C.byref(desc), arr, C.c_void_p(stream)), "otas_create")

    @classmethod
    def from_host_weights(cls, L, D, H, F, dtype, ln_eps, n_lead, layers_host, stream=None) -> "Context":
        """Upload per-layer dicts of host (NumPy float32) arrays to the GPU in the model's dtype and
        create the context on them."""
        import torch
        tdt = torch.float32 if dtype == OTAS_F32 else torch.bfloat16
        dev = [{k: torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).to("cuda").to(tdt).contiguous()
                for k, v in w.items()} for w in layers_host]
        return cls(L, D, H, F, dtype, ln_eps, n_lead, dev, stream)

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            self._lib.otas_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- pure host helpers
    def otas_workspace_bytes(self, B: int, T0: int) -> int:
        return int(self._lib.otas_workspace_bytes(self._h, B, T0))

    def otas_merge_workspace_bytes(self, B: int, T: int) -> int:
        return int(self._lib.otas_merge_workspace_bytes(B, T))

    # -- device entry points
    def otas_prompt_prepend(self, tokens, tok_offsets, prompts, prompt_offsets, out) -> np.ndarray:
        B = len(tok_offsets) - 1
        ta, tp = _i32(tok_offsets)
        pa, pp = _i32(prompt_offsets)
        oo = np.zeros(B + 1, dtype=np.int32)
        _check(self._lib.otas_prompt_prepend(self._h, _ptr(tokens), tp, _ptr(prompts), pp, B, _ptr(out),
                                             oo.ctypes.data_as(_I32P)), "otas_prompt_prepend")
        return oo

    def otas_prompt_prepend_pool(self, tokens, tok_offsets, pool, prompt_first, prompt_count, out) -> np.ndarray:
        B = len(tok_offsets) - 1
        ta, tp = _i32(tok_offsets)
        fa, fp = _i32(prompt_first)
        ca, cp = _i32(prompt_count)
        oo = np.zeros(B + 1, dtype=np.int32)
        _check(self._lib.otas_prompt_prepend_pool(self._h, _ptr(tokens), tp, _ptr(pool),
                                                  0 if pool is None else int(pool.shape[0]), fp, cp, B, _ptr(out),
                                                  oo.ctypes.data_as(_I32P)), "otas_prompt_prepend_pool")
        return oo

    def otas_token_merge(self, x, metric, dm, sizes, offsets, r, workspace, x_out, sizes_out,
                         trace_src=None, trace_dst=None) -> np.ndarray:
        B = len(offsets) - 1
        oa, op = _i32(offsets)
        ra, rp = _i32(r)
        oo = np.zeros(B + 1, dtype=np.int32)
        _check(self._lib.otas_token_merge(self._h, _ptr(x), _ptr(metric), dm, _ptr(sizes), op, rp, B,
                                          _ptr(workspace), workspace.numel() * workspace.element_size(),
                                          _ptr(x_out), _ptr(sizes_out), oo.ctypes.data_as(_I32P),
                                          _ptr(trace_src), _ptr(trace_dst)), "otas_token_merge")
        return oo

    def otas_token_merge_static(self, x, metric, dm, sizes, offsets, r, x_out, sizes_out,
                                trace_src=None, trace_dst=None) -> np.ndarray:
        B = len(offsets) - 1
        oa, op = _i32(offsets)
        ra, rp = _i32(r)
        oo = np.zeros(B + 1, dtype=np.int32)
        _check(self._lib.otas_token_merge_static(self._h, _ptr(x), _ptr(metric), dm, _ptr(sizes), op, rp, B,
                                                 _ptr(x_out), _ptr(sizes_out), oo.ctypes.data_as(_I32P),
                                                 _ptr(trace_src), _ptr(trace_dst)), "otas_token_merge_static")
        return oo

    def otas_encoder_forward(self, x0, offsets, r, flags, workspace, x_out, sizes_out,
                             trace_src=None, trace_dst=None) -> np.ndarray:
        B = len(offsets) - 1
        oa, op = _i32(offsets)
        ra, rp = _i32(r)
        oo = np.zeros(B + 1, dtype=np.int32)
        _check(self._lib.otas_encoder_forward(self._h, _ptr(x0), op, rp, B, flags, _ptr(workspace),
                                              workspace.numel() * workspace.element_size(), _ptr(x_out),
                                              _ptr(sizes_out), oo.ctypes.data_as(_I32P), _ptr(trace_src),
                                              _ptr(trace_dst)), "otas_encoder_forward")
        return oo

    def otas_encoder_layers(self, layer_begin, layer_end, x0, sizes_in, offsets, r, flags, workspace, x_out,
                            sizes_out, trace_src=None, trace_dst=None) -> np.ndarray:
        B = len(offsets) - 1
        oa, op = _i32(offsets)
        ra, rp = _i32(r)
        oo = np.zeros(B + 1, dtype=np.int32)
        _check(self._lib.otas_encoder_layers(self._h, layer_begin, layer_end, _ptr(x0), _ptr(sizes_in), op, rp, B,
                                             flags, _ptr(workspace), workspace.numel() * workspace.element_size(),
                                             _ptr(x_out), _ptr(sizes_out), oo.ctypes.data_as(_I32P),
                                             _ptr(trace_src), _ptr(trace_dst)), "otas_encoder_layers")
        return oo

    def otas_encoder_forward_deep(self, x0, offsets, mode, prompts, prompt_offsets, workspace, x_out,
                                  sizes_out) -> np.ndarray:
        """Per-layer prompting (mode OTAS_PROMPT_REPLACE / OTAS_PROMPT_GROW); prompts [L, P, D]."""
        B = len(offsets) - 1
        oa, op = _i32(offsets)
        pa, pp = _i32(prompt_offsets)
        oo = np.zeros(B + 1, dtype=np.int32)
        _check(self._lib.otas_encoder_forward_deep(self._h, _ptr(x0), op, B, int(mode), _ptr(prompts), pp,
                                                   _ptr(workspace), workspace.numel() * workspace.element_size(),
                                                   _ptr(x_out), _ptr(sizes_out), oo.ctypes.data_as(_I32P)),
               "otas_encoder_forward_deep")
        return oo

    def otas_patch_embed_workspace_bytes(self, B, C, Hi, Wi, patch) -> int:
        return int(self._lib.otas_patch_embed_workspace_bytes(self._h, B, C, Hi, Wi, patch))

    def otas_patch_embed(self, images, patch, w_patch, b_patch, cls, pos, workspace, tokens) -> np.ndarray:
        """images [B, C, Hi, Wi] -> tokens [B (n_lead + N), D]; returns the token offsets."""
        B, Cc, Hi, Wi = images.shape
        off = np.zeros(B + 1, dtype=np.int32)
        _check(self._lib.otas_patch_embed(self._h, _ptr(images), B, Cc, Hi, Wi, int(patch), _ptr(w_patch), _ptr(b_patch),
                                          _ptr(cls), _ptr(pos), _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _ptr(tokens),
                                          off.ctypes.data_as(_I32P)), "otas_patch_embed")
        return off

    def otas_task_heads(self, x, offsets, task, heads, lnf_g, lnf_b, logits) -> None:
        """heads: list of (w [K, D], b [K]) device tensors; logits [B, k_max] float32."""
        B = len(offsets) - 1
        oa, op = _i32(offsets)
        ta, tp = _i32(task)
        arr = (_TaskHead * len(heads))()
        for i, (w, b) in enumerate(heads):
            arr[i].w, arr[i].b, arr[i].classes = w.data_ptr(), b.data_ptr(), int(w.shape[0])
        _check(self._lib.otas_task_heads(self._h, _ptr(x), op, tp, B, arr, len(heads), _ptr(lnf_g), _ptr(lnf_b),
                                         _ptr(logits), int(logits.shape[1])), "otas_task_heads")

    def otas_layer_norm(self, x, g, b, T, y) -> None:
        _check(self._lib.otas_layer_norm(self._h, _ptr(x), _ptr(g), _ptr(b), T, _ptr(y)), "otas_layer_norm")

    def otas_linear(self, x, w, b, res, T, N, K, epilogue, y) -> None:
        _check(self._lib.otas_linear(self._h, _ptr(x), _ptr(w), _ptr(b), _ptr(res), T, N, K, epilogue, _ptr(y)),
               "otas_linear")

    def otas_linear_kernel(self, kernel, x, w, b, res, T, N, K, epilogue, y) -> None:
        _check(self._lib.otas_linear_kernel(self._h, int(kernel), _ptr(x), _ptr(w), _ptr(b), _ptr(res), T, N, K,
                                            epilogue, _ptr(y)), "otas_linear_kernel")

    def otas_linear_choice(self, T, N, K, epilogue) -> int:
        return int(self._lib.otas_linear_choice(self._h, int(T), int(N), int(K), int(epilogue)))

    def otas_attention(self, qkv, sizes, offsets, flags, o) -> None:
        B = len(offsets) - 1
        oa, op = _i32(offsets)
        _check(self._lib.otas_attention(self._h, _ptr(qkv), _ptr(sizes), op, B, flags, _ptr(o)), "otas_attention")

    def otas_timing_enable(self, on: bool) -> None:
        _check(self._lib.otas_timing_enable(self._h, 1 if on else 0), "otas_timing_enable")

    def otas_timing_read(self) -> dict:
        """{kind name: (total ms, launches)} since the last read."""
        k = self._lib.otas_timing_kinds()
        ms = (C.c_double * k)()
        cnt = (C.c_int64 * k)()
        _check(self._lib.otas_timing_read(self._h, ms, cnt), "otas_timing_read")
        return {self._lib.otas_timing_kind_name(i).decode(): (ms[i], int(cnt[i])) for i in range(k)}

    def otas_timing_kind_names(self) -> List[str]:
        return [self._lib.otas_timing_kind_name(i).decode() for i in range(self._lib.otas_timing_kinds())]

    def otas_splitk_room(self, T0: int, M: int) -> int:
        return int(self._lib.otas_splitk_room(self._h, int(T0), int(M)))

    def otas_splitk_factor(self, M: int, N: int, K: int, max_split: int = 8) -> int:
        return int(self._lib.otas_splitk_factor(self._h, int(M), int(N), int(K), int(max_split)))

    def otas_set_lanes(self, lanes: int) -> None:
        _check(self._lib.otas_set_lanes(self._h, int(lanes)), "otas_set_lanes")

    def otas_clock_probe_start(self, samples: int) -> None:
        _check(self._lib.otas_clock_probe_start(self._h, int(samples)), "otas_clock_probe_start")

    def otas_clock_probe_read(self, cap: int = 65536) -> List[float]:
        """Shader clock in MHz of every sample of the probe started last, in order (waits for the probe)."""
        mhz = (C.c_float * cap)()
        n = C.c_int32(0)
        _check(self._lib.otas_clock_probe_read(self._h, mhz, cap, C.byref(n)), "otas_clock_probe_read")
        return [float(mhz[i]) for i in range(n.value)]

    def otas_timing_overhead_ms(self) -> float:
        return float(self._lib.otas_timing_overhead_ms(self._h))

    def otas_timing_read_launches(self, cap: int = 65536):
        """[(kind name, ms)] of the recorded launches in launch order (records are kept)."""
        kinds = (C.c_int32 * cap)()
        ms = (C.c_float * cap)()
        n = self._lib.otas_timing_read_launches(self._h, cap, kinds, ms)
        if n < 0:
            raise OtasError(4, "otas_timing_read_launches")
        return [(self._lib.otas_timing_kind_name(kinds[i]).decode(), float(ms[i])) for i in range(min(n, cap))]

    # -- plan arithmetic shared with callers (host only)
    def trace_layout(self, lengths0: Sequence[int], r: Sequence[int],
                     n_layers: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
        """(r_eff[n_layers][B], trace_offset[n_layers][B]) of the trace buffers of
        otas_encoder_forward / otas_encoder_layers, from the library's own schedule function."""
        B = len(lengths0)
        nl = self.L if n_layers is None else n_layers
        reff = np.zeros((nl, B), dtype=np.int64)
        for q in range(B):
            s = otas_schedule(int(lengths0[q]), 0, int(r[q]), self.n_lead, nl)
            reff[:, q] = -np.diff(np.asarray(s))
        flat = reff.reshape(-1)
        troff = np.concatenate([[0], np.cumsum(flat)[:-1]]).reshape(nl, B)
        return reff, troff


def otas_sched_rate_table(gammas: Sequence[int], latency) -> List[Tuple[float, int]]:
    """otas_sched_rate_table: rows (largest request rate, index into gammas) of the projection f of Alg. 3
    from a latency profile [n_tasks][len(gammas)]."""
    lat = np.ascontiguousarray(np.asarray(latency, dtype=np.float64))
    if lat.ndim != 2 or lat.shape[1] != len(gammas):
        raise ValueError("latency must be [n_tasks][len(gammas)]")
    ga, gp = _i32(gammas)
    rm = np.zeros(max(len(gammas), 1), dtype=np.float64)
    rg = np.zeros(max(len(gammas), 1), dtype=np.int32)
    n = C.c_int32()
    _check(load_library().otas_sched_rate_table(len(gammas), gp, lat.shape[0], lat.ctypes.data_as(_F64P),
                                                rm.ctypes.data_as(_F64P), rg.ctypes.data_as(_I32P), C.byref(n)),
           "otas_sched_rate_table")
    return [(float(rm[i]), int(rg[i])) for i in range(n.value)]


class Scheduler:
    """Handle of an otas_sched object (include/otas_sched.h): batch queue, adaptive batching, token
    adaptation.  Host only; the methods carry the C names and marshal arguments."""

    def __init__(self, gammas: Sequence[int], latency, accuracy, rate_table: Sequence[Tuple[float, int]] = (),
                 delta: float = 0.5, epsilon: int = 64, eta: float = 0.5, mu: float = 0.8, beta: int = 5,
                 kappa: float = 0.8):
        """otas_sched_create.  latency / accuracy: [n_tasks][len(gammas)]; rate_table: rows of (largest
        request rate, index into gammas), ascending.  The defaults are the paper's settings (Sec. V)."""
        self._lib = load_library()
        self._h = C.c_void_p()
        lat = np.ascontiguousarray(np.asarray(latency, dtype=np.float64))
        acc = np.ascontiguousarray(np.asarray(accuracy, dtype=np.float64))
        if lat.ndim != 2 or lat.shape != acc.shape or lat.shape[1] != len(gammas):
            raise ValueError("latency and accuracy must be [n_tasks][len(gammas)]")
        self.gammas = [int(g) for g in gammas]
        ga, gp = _i32(self.gammas)
        rm = np.ascontiguousarray(np.asarray([r[0] for r in rate_table], dtype=np.float64))
        rg, rgp = _i32([r[1] for r in rate_table])
        prm = _SchedParams(delta, eta, mu, kappa, epsilon, beta)
        _check(self._lib.otas_sched_create(C.byref(prm), len(self.gammas), gp, lat.shape[0],
                                           lat.ctypes.data_as(_F64P), acc.ctypes.data_as(_F64P), len(rate_table),
                                           rm.ctypes.data_as(_F64P) if len(rate_table) else None,
                                           rgp if len(rate_table) else None, C.byref(self._h)), "otas_sched_create")

    def otas_sched_destroy(self) -> None:
        if self._h:
            self._lib.otas_sched_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.otas_sched_destroy()
        except Exception:
            pass

    def otas_sched_add_query(self, id: int, s_r: float, l_r: float, u_r: float, task: int) -> int:
        b = C.c_int32()
        _check(self._lib.otas_sched_add_query(self._h, int(id), s_r, l_r, u_r, int(task), C.byref(b)),
               "otas_sched_add_query")
        return b.value

    def otas_sched_allocate(self, T: float, q: float, initial_stage: bool) -> float:
        out = C.c_double()
        _check(self._lib.otas_sched_allocate(self._h, T, q, 1 if initial_stage else 0, C.byref(out)),
               "otas_sched_allocate")
        return out.value

    def otas_sched_num_batches(self) -> int:
        return int(self._lib.otas_sched_num_batches(self._h))

    def otas_sched_batch_info(self, b: int) -> dict:
        n, g = C.c_int32(), C.c_int32()
        s_b, d_b, u_b = C.c_double(), C.c_double(), C.c_double()
        _check(self._lib.otas_sched_batch_info(self._h, int(b), C.byref(n), C.byref(s_b), C.byref(d_b), C.byref(u_b),
                                               C.byref(g)), "otas_sched_batch_info")
        return {"size": n.value, "s_b": s_b.value, "d_b": d_b.value, "u_b": u_b.value, "gamma_index": g.value}

    def otas_sched_batch_queries(self, b: int) -> Tuple[List[int], List[int]]:
        n = C.c_int32()
        _check(self._lib.otas_sched_batch_queries(self._h, int(b), None, None, 0, C.byref(n)),
               "otas_sched_batch_queries")
        ids = (C.c_int64 * max(n.value, 1))()
        tasks = (C.c_int32 * max(n.value, 1))()
        _check(self._lib.otas_sched_batch_queries(self._h, int(b), ids, tasks, n.value, None),
               "otas_sched_batch_queries")
        return list(ids[:n.value]), list(tasks[:n.value])

    def otas_sched_estimate(self, b: int, gamma_index: int) -> Tuple[float, float]:
        t, U = C.c_double(), C.c_double()
        _check(self._lib.otas_sched_estimate(self._h, int(b), int(gamma_index), C.byref(t), C.byref(U)),
               "otas_sched_estimate")
        return t.value, U.value

    def otas_sched_remove(self, b: int) -> None:
        _check(self._lib.otas_sched_remove(self._h, int(b)), "otas_sched_remove")
