"""ctypes binding of libkeep_hip.so: argument marshalling only.

Every step of the path runs inside the library's HIP kernels; this module turns
torch tensors (device memory, streams) and Python lists into the plain pointers
and sizes of include/keep.h and raises KeepError on a non-zero status.  There is
no CPU fallback: loading fails loudly when the library has not been built.
"""
import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libkeep_hip.so")

KEEP_OK = 0
KEEP_ERR_INVALID_ARG, KEEP_ERR_SHAPE, KEEP_ERR_STATE, KEEP_ERR_WORKSPACE, KEEP_ERR_HIP, KEEP_ERR_UNSUPPORTED = range(1, 7)
KEEP_F32, KEEP_BF16 = 0, 1
KEEP_KV_DEVICE, KEEP_KV_PINNED_HOST = 0, 1
KEEP_BUDGET_GROUP_COUNT, KEEP_BUDGET_TOKENS = 0, 1
KEEP_LOAD_SERIAL, KEEP_LOAD_NEXT_LAYER, KEEP_LOAD_LAYER_BALANCED = 0, 1, 2
KEEP_KERNELS_AUTO, KEEP_KERNELS_GENERIC = 0, 1
KEEP_REPORT_MAX_LAYERS = 128

KEEP_OPT_PROPAGATION_SOURCES = 0
KEEP_SOURCES_QUERY_AND_SET, KEEP_SOURCES_SET_ONLY = 0, 1
KEEP_STATE_ATTN_OUT, KEEP_STATE_LSE = 0, 1

EXPORTED = ("keep_init", "keep_destroy", "keep_last_error", "keep_uses_mfma", "keep_workspace_bytes", "keep_recompute_layer",
            "keep_set_option", "keep_read_layer_state", "keep_select_groups_static", "keep_prefill_tokens",
            "keep_select_tokens",
            "keep_score_groups", "keep_select_groups", "keep_prefill",
            "keep_prefill_padded", "keep_decode", "keep_precompute_group", "keep_precompute_groups",
            "keep_dequantize_int4", "keep_attach_int4",
            "keep_memory_create", "keep_memory_destroy", "keep_memory_last_error",
            "keep_memory_put", "keep_memory_remove", "keep_memory_end_step", "keep_memory_unit_count",
            "keep_memory_unit_info", "keep_memory_unit_tokens", "keep_memory_mark_computed")


class KeepError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("keep status %d: %s" % (status, text))
        self.status = status


class ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn_dim", "vocab")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float)] + \
               [(n, C.c_int32) for n in ("dtype", "max_tokens", "max_groups", "kernel_path")]


_W_NAMES = ("ln1", "wq", "wk", "wv", "bq", "bk", "bv", "wo", "ln2", "wgate", "wup", "wdown")


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _W_NAMES]


_W4_NAMES = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")


class Int4Matrix(C.Structure):
    _fields_ = [("codes", C.c_void_p), ("scale_zero", C.c_void_p)]


class LayerWeightsInt4(C.Structure):
    _fields_ = [(n, Int4Matrix) for n in _W4_NAMES]


class Prompt(C.Structure):
    _fields_ = [("n_groups", C.c_int32), ("group_len", C.POINTER(C.c_int32)), ("group_kind", C.POINTER(C.c_uint8)),
                ("instr_len", C.c_int32), ("token_ids", C.POINTER(C.c_int32)),
                ("k_blocks", C.POINTER(C.c_void_p)), ("v_blocks", C.POINTER(C.c_void_p)), ("kv_location", C.c_int32)]


_L = KEEP_REPORT_MAX_LAYERS
_REPORT_MS = ("ms_realign", "ms_prep", "ms_qkv_gemm", "ms_rope", "ms_attn", "ms_oproj", "ms_norm2", "ms_gateup",
              "ms_down", "ms_score")


class Report(C.Structure):
    _fields_ = ([("events_in", C.c_int32), ("n_layers", C.c_int32), ("used_mfma", C.c_int32), ("ms_total", C.c_float),
                 ("rows", C.c_int32 * _L), ("set_size", C.c_int32 * _L), ("hops_run", C.c_int32 * _L),
                 ("realign_rows", C.c_int32 * _L), ("ffn_rows", C.c_int32 * _L),
                 ("attn_rows", C.c_int32 * _L), ("attn_keys", C.c_uint64 * _L)]
                + [(_n, C.c_float * _L) for _n in _REPORT_MS]
                + [("bytes_loaded", C.c_uint64 * _L)])


_lib = None


class MemoryUnit(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("kind", "id", "group", "n_segments", "n_tokens", "dirty")]


class MemoryStepReport(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("step", "n_static", "n_dynamic", "n_to_dynamic", "n_to_static",
                                         "dirty_units")] + [("dirty_tokens", C.c_int64)]


def load_library() -> C.CDLL:
    """dlopen the HIP library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libkeep_hip.so is missing: build it with `python -m paper_2602_23592_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, f32 = C.c_void_p, C.c_int32, C.c_float
    pi32 = C.POINTER(C.c_int32)
    lib.keep_init.restype = i32
    lib.keep_init.argtypes = [C.POINTER(ModelDesc), C.POINTER(LayerWeights), vp, vp, vp, vp, C.POINTER(vp)]
    lib.keep_destroy.restype = i32
    lib.keep_destroy.argtypes = [vp]
    lib.keep_last_error.restype = C.c_char_p
    lib.keep_last_error.argtypes = [vp]
    lib.keep_uses_mfma.restype = i32
    lib.keep_uses_mfma.argtypes = [vp]
    lib.keep_workspace_bytes.restype = C.c_uint64
    lib.keep_workspace_bytes.argtypes = [C.POINTER(ModelDesc)]
    lib.keep_set_option.restype = i32
    lib.keep_set_option.argtypes = [vp, i32, i32]
    lib.keep_read_layer_state.restype = i32
    lib.keep_read_layer_state.argtypes = [vp, i32, vp, C.c_uint64]
    lib.keep_recompute_layer.restype = i32
    lib.keep_recompute_layer.argtypes = [vp, C.POINTER(Prompt), i32, pi32, i32, vp, vp, vp, vp]
    lib.keep_score_groups.restype = i32
    lib.keep_score_groups.argtypes = [vp, C.POINTER(Prompt), i32, pi32, i32, f32, i32, i32, C.POINTER(f32), pi32, pi32, pi32]
    lib.keep_select_groups.restype = i32
    lib.keep_select_groups.argtypes = [vp, C.POINTER(f32), pi32, i32, pi32, i32, f32, i32, i32, pi32, pi32, pi32]
    lib.keep_select_groups_static.restype = i32
    lib.keep_select_groups_static.argtypes = [vp, vp, i32, vp, i32, i32, f32, i32, i32, i32, vp, vp]
    lib.keep_prefill_tokens.restype = i32
    lib.keep_prefill_tokens.argtypes = [vp, C.POINTER(Prompt), C.POINTER(f32), i32, vp, vp, vp, pi32, pi32,
                                        C.POINTER(f32), C.POINTER(Report)]
    lib.keep_select_tokens.restype = i32
    lib.keep_select_tokens.argtypes = [vp, C.POINTER(f32), i32, i32, pi32]
    lib.keep_prefill.restype = i32
    lib.keep_prefill.argtypes = [vp, C.POINTER(Prompt), C.POINTER(f32), i32, i32, i32, vp, vp, vp, pi32, pi32,
                                 C.POINTER(Report)]
    lib.keep_prefill_padded.restype = i32
    lib.keep_prefill_padded.argtypes = [vp, C.POINTER(Prompt), C.POINTER(f32), i32, i32, i32, vp, vp, i32, vp, pi32, pi32,
                                        C.POINTER(Report)]
    lib.keep_decode.restype = i32
    lib.keep_decode.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, pi32, vp, pi32]
    lib.keep_dequantize_int4.restype = i32
    lib.keep_dequantize_int4.argtypes = [vp, vp, i32, i32, vp, vp]
    lib.keep_attach_int4.restype = i32
    lib.keep_attach_int4.argtypes = [vp, C.POINTER(LayerWeightsInt4)]
    lib.keep_precompute_group.restype = i32
    lib.keep_precompute_group.argtypes = [vp, pi32, i32, vp, vp, C.POINTER(Report)]
    lib.keep_precompute_groups.restype = i32
    lib.keep_precompute_groups.argtypes = [vp, i32, pi32, pi32, vp, vp, C.POINTER(Report)]
    lib.keep_memory_create.restype = i32
    lib.keep_memory_create.argtypes = [i32, C.POINTER(vp)]
    lib.keep_memory_destroy.restype = i32
    lib.keep_memory_destroy.argtypes = [vp]
    lib.keep_memory_last_error.restype = C.c_char_p
    lib.keep_memory_last_error.argtypes = [vp]
    lib.keep_memory_put.restype = i32
    lib.keep_memory_put.argtypes = [vp, i32, i32, pi32, i32, pi32]
    lib.keep_memory_remove.restype = i32
    lib.keep_memory_remove.argtypes = [vp, i32]
    lib.keep_memory_end_step.restype = i32
    lib.keep_memory_end_step.argtypes = [vp, C.POINTER(MemoryStepReport), pi32, i32, pi32, i32]
    lib.keep_memory_unit_count.restype = i32
    lib.keep_memory_unit_count.argtypes = [vp]
    lib.keep_memory_unit_info.restype = i32
    lib.keep_memory_unit_info.argtypes = [vp, i32, C.POINTER(MemoryUnit)]
    lib.keep_memory_unit_tokens.restype = i32
    lib.keep_memory_unit_tokens.argtypes = [vp, i32, pi32, i32, pi32]
    lib.keep_memory_mark_computed.restype = i32
    lib.keep_memory_mark_computed.argtypes = [vp, i32]
    _lib = lib
    return lib


def _i32_array(values: Sequence[int]):
    a = np.ascontiguousarray(np.asarray(values, dtype=np.int32))
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream_handle(s) -> Optional[int]:
    if s is None:
        return None
    return s.cuda_stream if hasattr(s, "cuda_stream") else int(s)


class KeepPrompt:
    """Keeps the host arrays of a keep_prompt alive and exposes the C struct."""

    def __init__(self, group_len: Sequence[int], instr_len: int, token_ids: Sequence[int], k_blocks, v_blocks,
                 n_layers: int, kv_location: int = KEEP_KV_DEVICE, group_kind: Optional[Sequence[int]] = None):
        self.group_len = [int(v) for v in group_len]
        self.instr_len = int(instr_len)
        self.n_groups = len(self.group_len)
        self._gl, gl_p = _i32_array(self.group_len if self.n_groups else [0])
        self._tok, tok_p = _i32_array(token_ids)
        self._kind = None
        kind_p = None
        if group_kind is not None:
            self._kind = np.ascontiguousarray(np.asarray(group_kind, dtype=np.uint8))
            kind_p = self._kind.ctypes.data_as(C.POINTER(C.c_uint8))
        # k_blocks[l][g]: tensors (device or pinned host); flattened to layer*G + g
        self._blocks = (k_blocks, v_blocks)     # keep the tensors alive
        n = max(1, n_layers * self.n_groups)
        self._kp = (C.c_void_p * n)()
        self._vp = (C.c_void_p * n)()
        if k_blocks is not None:
            for l in range(n_layers):
                for g in range(self.n_groups):
                    self._kp[l * self.n_groups + g] = k_blocks[l][g].data_ptr()
                    self._vp[l * self.n_groups + g] = v_blocks[l][g].data_ptr()
        self.c = Prompt(self.n_groups, gl_p, kind_p, self.instr_len, tok_p,
                        C.cast(self._kp, C.POINTER(C.c_void_p)), C.cast(self._vp, C.POINTER(C.c_void_p)), kv_location)

    @property
    def n_mem(self) -> int:
        return sum(self.group_len)

    @property
    def n_tokens(self) -> int:
        return self.n_mem + self.instr_len

    def n_rows(self, groups: Sequence[int]) -> int:
        return sum(self.group_len[g] for g in groups) + self.instr_len


def dequantize_int4(codes: torch.Tensor, scale_zero: torch.Tensor, rows: int, k: int, stream=None) -> torch.Tensor:
    """keep_dequantize_int4: codes (uint8, rows * K / 2) and scale_zero (32-bit words, rows * K / 128) in the
    library's block order, on the device -> the bfloat16 weights [rows, K] (new device tensor; the allocation is
    the only thing done here)."""
    lib = load_library()
    assert codes.is_cuda and codes.is_contiguous() and codes.dtype == torch.uint8 and codes.numel() == rows * k // 2
    assert scale_zero.is_cuda and scale_zero.is_contiguous() and scale_zero.element_size() == 4
    assert scale_zero.numel() == rows * k // 128
    out = torch.empty((rows, k), dtype=torch.bfloat16, device=codes.device)
    st = lib.keep_dequantize_int4(codes.data_ptr(), scale_zero.data_ptr(), rows, k, out.data_ptr(),
                                  _stream_handle(stream if stream is not None else torch.cuda.current_stream()))
    if st != KEEP_OK:
        raise KeepError(st, lib.keep_last_error(None).decode())
    return out


def select_groups_static(S: torch.Tensor, groups: torch.Tensor, group_len: torch.Tensor, mem_tokens: int,
                         ratio_next: float, hops: int, budget_mode: int, propagation_sources: int,
                         result: torch.Tensor, stream=None):
    """keep_select_groups_static: every tensor is caller-allocated device memory (S float32 [(m+1), m], groups
    int32 [m], group_len int32 [G], result int32 [m + 2]); nothing is allocated here or in the library."""
    lib = load_library()
    m = int(groups.numel())
    for t, dt in ((S, torch.float32), (groups, torch.int32), (group_len, torch.int32), (result, torch.int32)):
        assert t.is_cuda and t.is_contiguous() and t.dtype == dt
    assert S.numel() == (m + 1) * m and result.numel() >= m + 2
    st = lib.keep_select_groups_static(S.data_ptr(), groups.data_ptr(), m, group_len.data_ptr(), int(group_len.numel()),
                                       int(mem_tokens), float(ratio_next), hops, budget_mode, propagation_sources,
                                       result.data_ptr(),
                                       _stream_handle(stream if stream is not None else torch.cuda.current_stream()))
    if st != KEEP_OK:
        raise KeepError(st, lib.keep_last_error(None).decode())


class KeepContext:
    """keep_ctx handle.  Weights: list of dicts name -> device tensor (or None for absent biases)."""

    def __init__(self, shape, layers: List[dict], embed: torch.Tensor, max_tokens: int, max_groups: int,
                 kernel_path: int = KEEP_KERNELS_AUTO, stream_compute=None, stream_eval=None, stream_copy=None):
        self.lib = load_library()
        self.shape = shape
        self.dtype = KEEP_BF16 if shape.storage == "bf16" else KEEP_F32
        self.torch_dtype = torch.bfloat16 if shape.storage == "bf16" else torch.float32
        self.desc = ModelDesc(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                              shape.ffn_dim, shape.vocab, shape.rope_theta, shape.rms_eps, self.dtype,
                              int(max_tokens), int(max_groups), kernel_path)
        self._keep = (layers, embed, stream_compute, stream_eval, stream_copy)
        arr = (LayerWeights * shape.n_layers)()
        for l, w in enumerate(layers):
            for n in _W_NAMES:
                t = w.get(n)
                if t is not None:
                    assert t.is_cuda and t.is_contiguous() and t.dtype == self.torch_dtype, n
                setattr(arr[l], n, _ptr(t))
        assert embed.is_cuda and embed.is_contiguous() and embed.dtype == self.torch_dtype
        self.device = embed.device
        handle = C.c_void_p()
        st = self.lib.keep_init(C.byref(self.desc), arr, embed.data_ptr(), _stream_handle(stream_compute),
                                _stream_handle(stream_eval), _stream_handle(stream_copy), C.byref(handle))
        if st != KEEP_OK:
            raise KeepError(st, self.lib.keep_last_error(None).decode())
        self.handle = handle

    def close(self):
        if getattr(self, "handle", None):
            self.lib.keep_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def attach_int4(self, layers4: Optional[List[dict]]):
        """keep_attach_int4.  layers4: per layer a dict name -> (codes, scale_zero) device tensors for the seven
        projections, or None to detach.  The tensors are kept alive by this object."""
        if layers4 is None:
            self._check(self.lib.keep_attach_int4(self.handle, None))
            self._keep4 = None
            return
        arr = (LayerWeightsInt4 * self.shape.n_layers)()
        for l, w in enumerate(layers4):
            for n in _W4_NAMES:
                codes, sz = w[n][0], w[n][1]
                assert codes.is_cuda and codes.is_contiguous() and sz.is_cuda and sz.is_contiguous(), n
                getattr(arr[l], n).codes = codes.data_ptr()
                getattr(arr[l], n).scale_zero = sz.data_ptr()
        self._check(self.lib.keep_attach_int4(self.handle, arr))
        self._keep4 = layers4

    @property
    def uses_mfma(self) -> bool:
        return self.lib.keep_uses_mfma(self.handle) == 1

    def _check(self, st: int):
        if st != KEEP_OK:
            raise KeepError(st, self.lib.keep_last_error(self.handle).decode())

    # -- the C entry points ---------------------------------------------------
    def set_option(self, option: int, value: int):
        self._check(self.lib.keep_set_option(self.handle, option, value))

    def read_layer_state(self, what: int, n_rows: int) -> np.ndarray:
        """keep_read_layer_state: attention output [n_rows, Hq, dh] (float32 view of the stored values) or
        log-sum-exp [n_rows, Hq] of the last keep_recompute_layer, on the host."""
        s = self.shape
        if what == KEEP_STATE_LSE:
            out = np.empty((n_rows, s.n_q_heads), dtype=np.float32)
        elif self.dtype == KEEP_BF16:
            out = np.empty((n_rows, s.n_q_heads, s.head_dim), dtype=np.uint16)
        else:
            out = np.empty((n_rows, s.n_q_heads, s.head_dim), dtype=np.float32)
        self._check(self.lib.keep_read_layer_state(self.handle, what, out.ctypes.data_as(C.c_void_p), out.nbytes))
        if out.dtype == np.uint16:      # bfloat16 bit patterns -> the float32 values they stand for
            out = (out.astype(np.uint32) << np.uint32(16)).view(np.float32)
        return out

    def recompute_layer(self, prompt: KeepPrompt, layer: int, groups: Sequence[int], x_in: Optional[torch.Tensor],
                        x_out: torch.Tensor, k_cache_l: torch.Tensor, v_cache_l: torch.Tensor):
        g, gp = _i32_array(groups if len(groups) else [0])
        self._check(self.lib.keep_recompute_layer(self.handle, C.byref(prompt.c), layer, gp, len(groups), _ptr(x_in),
                                                  x_out.data_ptr(), k_cache_l.data_ptr(), v_cache_l.data_ptr()))

    def score_groups(self, prompt: KeepPrompt, layer: int, groups: Sequence[int], ratio_next: float, hops: int,
                     budget_mode: int = KEEP_BUDGET_GROUP_COUNT, want_scores: bool = True):
        m = len(groups)
        g, gp = _i32_array(groups if m else [0])
        S = np.zeros((m + 1, max(m, 1)), dtype=np.float32) if want_scores else None
        nxt = np.zeros(max(m, 1), dtype=np.int32)
        n_next, runs = C.c_int32(0), C.c_int32(0)
        self._check(self.lib.keep_score_groups(
            self.handle, C.byref(prompt.c), layer, gp, m, float(ratio_next), hops, budget_mode,
            S.ctypes.data_as(C.POINTER(C.c_float)) if want_scores else None,
            nxt.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(n_next), C.byref(runs)))
        scores = S[:, :m].reshape(m + 1, m) if want_scores else None
        return [int(v) for v in nxt[:n_next.value]], runs.value, scores

    def select_groups(self, S: np.ndarray, groups: Sequence[int], group_len: Sequence[int], ratio_next: float,
                      hops: int, budget_mode: int = KEEP_BUDGET_GROUP_COUNT):
        m = len(groups)
        S = np.ascontiguousarray(S, dtype=np.float32)
        assert S.shape == (m + 1, m)
        g, gp = _i32_array(groups if m else [0])
        gl, glp = _i32_array(group_len if len(group_len) else [0])
        nxt = np.zeros(max(m, 1), dtype=np.int32)
        n_next, runs = C.c_int32(0), C.c_int32(0)
        self._check(self.lib.keep_select_groups(
            self.handle, S.ctypes.data_as(C.POINTER(C.c_float)), gp, m, glp, len(group_len), float(ratio_next), hops,
            budget_mode, nxt.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(n_next), C.byref(runs)))
        return [int(v) for v in nxt[:n_next.value]], runs.value

    def prefill(self, prompt: KeepPrompt, ratios: Sequence[float], hops: int, k_cache: torch.Tensor,
                v_cache: torch.Tensor, x_final: torch.Tensor, budget_mode: int = KEEP_BUDGET_GROUP_COUNT,
                load_mode: int = KEEP_LOAD_LAYER_BALANCED, want_report: bool = False,
                cache_rows: Optional[int] = None, gate_up_events_only: bool = False):
        """cache_rows: rows per layer of k_cache / v_cache when they leave room for decoded tokens.
        gate_up_events_only: with a report, time only the gate/up GEMM (far fewer HIP events in the stream)."""
        L, G = self.shape.n_layers, prompt.n_groups
        r = np.ascontiguousarray(np.asarray(ratios, dtype=np.float32))
        sel = np.zeros(max(1, L * G), dtype=np.int32)
        cnt = np.zeros(L, dtype=np.int32)
        rep = Report() if want_report else None
        if want_report:
            rep.events_in = 1 if gate_up_events_only else 0
        if cache_rows is None:
            self._check(self.lib.keep_prefill(
                self.handle, C.byref(prompt.c), r.ctypes.data_as(C.POINTER(C.c_float)), hops, budget_mode, load_mode,
                k_cache.data_ptr(), v_cache.data_ptr(), x_final.data_ptr(), sel.ctypes.data_as(C.POINTER(C.c_int32)),
                cnt.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(rep) if want_report else None))
        else:
            self._check(self.lib.keep_prefill_padded(
                self.handle, C.byref(prompt.c), r.ctypes.data_as(C.POINTER(C.c_float)), hops, budget_mode, load_mode,
                k_cache.data_ptr(), v_cache.data_ptr(), cache_rows, x_final.data_ptr(),
                sel.ctypes.data_as(C.POINTER(C.c_int32)), cnt.ctypes.data_as(C.POINTER(C.c_int32)),
                C.byref(rep) if want_report else None))
        sets = [[int(v) for v in sel[l * G:l * G + cnt[l]]] for l in range(L)]
        return sets, rep

    def prefill_tokens(self, prompt: KeepPrompt, ratios: Sequence[float], k_cache: torch.Tensor, v_cache: torch.Tensor,
                       x_final: torch.Tensor, load_mode: int = KEEP_LOAD_LAYER_BALANCED, want_deviation: bool = False,
                       want_report: bool = False):
        """keep_prefill_tokens.  Returns (rows per layer, deviations per layer or None, report or None)."""
        L, nm = self.shape.n_layers, prompt.n_mem
        r = np.ascontiguousarray(np.asarray(ratios, dtype=np.float32))
        sel = np.zeros(max(1, L * nm), dtype=np.int32)
        cnt = np.zeros(L, dtype=np.int32)
        dev = np.zeros(max(1, L * nm), dtype=np.float32) if want_deviation else None
        rep = Report() if want_report else None
        self._check(self.lib.keep_prefill_tokens(
            self.handle, C.byref(prompt.c), r.ctypes.data_as(C.POINTER(C.c_float)), load_mode, k_cache.data_ptr(),
            v_cache.data_ptr(), x_final.data_ptr(), sel.ctypes.data_as(C.POINTER(C.c_int32)),
            cnt.ctypes.data_as(C.POINTER(C.c_int32)),
            dev.ctypes.data_as(C.POINTER(C.c_float)) if want_deviation else None,
            C.byref(rep) if want_report else None))
        rows = [[int(v) for v in sel[l * nm:l * nm + cnt[l]]] for l in range(L)]
        devs = [dev[l * nm:l * nm + cnt[l]].copy() for l in range(L)] if want_deviation else None
        return rows, devs, rep

    def select_tokens(self, deviation: np.ndarray, k: int) -> List[int]:
        d = np.ascontiguousarray(deviation, dtype=np.float32)
        out = np.zeros(max(1, k), dtype=np.int32)
        self._check(self.lib.keep_select_tokens(self.handle, d.ctypes.data_as(C.POINTER(C.c_float)), len(d), k,
                                                out.ctypes.data_as(C.POINTER(C.c_int32))))
        return [int(v) for v in out[:k]]

    def precompute_groups(self, unit_len: Sequence[int], token_ids: Sequence[int], k_blocks: torch.Tensor,
                          v_blocks: torch.Tensor, want_report: bool = False):
        """KV blocks [n_layers][sum(unit_len), n_kv_heads, head_dim] of several units, each computed on its own."""
        ul, ulp = _i32_array(unit_len)
        ids, ip = _i32_array(token_ids)
        rep = Report() if want_report else None
        self._check(self.lib.keep_precompute_groups(self.handle, len(ul), ulp, ip, k_blocks.data_ptr(),
                                                    v_blocks.data_ptr(), C.byref(rep) if want_report else None))
        return rep

    def decode(self, final_norm: torch.Tensor, lm_head: torch.Tensor, x_last: torch.Tensor, k_cache: torch.Tensor,
               v_cache: torch.Tensor, n_ctx: int, n_new: int, logits_out: Optional[torch.Tensor] = None,
               forced_tokens: Optional[Sequence[int]] = None):
        """Greedy tokens after a prompt of n_ctx tokens; caches are [n_layers, cache_rows, Hkv, dh]."""
        out = np.zeros(max(1, n_new), dtype=np.int32)
        fp = None
        if forced_tokens is not None:
            f, fp = _i32_array(list(forced_tokens) if len(forced_tokens) else [0])
        self._check(self.lib.keep_decode(self.handle, final_norm.data_ptr(), lm_head.data_ptr(), x_last.data_ptr(),
                                         k_cache.data_ptr(), v_cache.data_ptr(), k_cache.shape[1], n_ctx, n_new,
                                         out.ctypes.data_as(C.POINTER(C.c_int32)), _ptr(logits_out), fp))
        return [int(v) for v in out[:n_new]]

    def precompute_group(self, token_ids: Sequence[int], k_blocks: torch.Tensor, v_blocks: torch.Tensor,
                         want_report: bool = False):
        """KV blocks [n_layers][n, n_kv_heads, head_dim] of one memory unit computed on its own."""
        ids, ip = _i32_array(token_ids)
        rep = Report() if want_report else None
        self._check(self.lib.keep_precompute_group(self.handle, ip, len(ids), k_blocks.data_ptr(), v_blocks.data_ptr(),
                                                   C.byref(rep) if want_report else None))
        return rep


class KeepMemory:
    """Static-dynamic memory store of the library (host-side bookkeeping; marshalling only)."""

    def __init__(self, window_t: int):
        self.lib = load_library()
        h = C.c_void_p()
        st = self.lib.keep_memory_create(window_t, C.byref(h))
        if st != KEEP_OK:
            raise KeepError(st, "keep_memory_create failed")
        self.handle = h

    def close(self):
        if self.handle:
            self.lib.keep_memory_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != KEEP_OK:
            raise KeepError(st, self.lib.keep_memory_last_error(self.handle).decode())

    def put(self, group: int, segment: int, tokens: Sequence[int]) -> bool:
        ids, ip = _i32_array(tokens if len(tokens) else [0])
        changed = C.c_int32(0)
        self._check(self.lib.keep_memory_put(self.handle, group, segment, ip, len(tokens), C.byref(changed)))
        return bool(changed.value)

    def remove(self, segment: int):
        self._check(self.lib.keep_memory_remove(self.handle, segment))

    def end_step(self, cap: int = 4096):
        rep = MemoryStepReport()
        td = np.zeros(cap, dtype=np.int32)
        ts = np.zeros(cap, dtype=np.int32)
        p32 = C.POINTER(C.c_int32)
        self._check(self.lib.keep_memory_end_step(self.handle, C.byref(rep), td.ctypes.data_as(p32), cap,
                                                  ts.ctypes.data_as(p32), cap))
        return rep, [int(v) for v in td[:rep.n_to_dynamic]], [int(v) for v in ts[:rep.n_to_static]]

    def units(self):
        out = []
        for i in range(self.lib.keep_memory_unit_count(self.handle)):
            u = MemoryUnit()
            self._check(self.lib.keep_memory_unit_info(self.handle, i, C.byref(u)))
            out.append(u)
        return out

    def unit_tokens(self, unit: int, cap: int):
        buf = np.zeros(max(1, cap), dtype=np.int32)
        n = C.c_int32(0)
        self._check(self.lib.keep_memory_unit_tokens(self.handle, unit, buf.ctypes.data_as(C.POINTER(C.c_int32)), cap,
                                                     C.byref(n)))
        return [int(v) for v in buf[:n.value]]

    def mark_computed(self, unit: int):
        self._check(self.lib.keep_memory_mark_computed(self.handle, unit))
