"""ctypes binding of libarb (include/arb.h): argument marshalling only.

Every step of the forward runs in the library's HIP kernels; torch is used for
device memory and for the current stream.  There is no fallback path: if the
shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libarb.so")
_lib = None

ARB_OK, ARB_EINVAL, ARB_ESHAPE, ARB_ECAPACITY, ARB_EHIP, ARB_EUNSUPPORTED = range(6)
ARB_POOL_MEAN, ARB_POOL_LAST = 0, 1
ARB_HEAD_NONE, ARB_HEAD_LINEAR, ARB_HEAD_TWO_CLASS = 0, 1, 2
ARB_ESCALATE_IF_GT, ARB_ACCEPT_IF_GT = 0, 1
ARB_EPI_STORE_BF16, ARB_EPI_RESIDUAL_F32, ARB_EPI_SWIGLU_BF16, ARB_EPI_STORE_F32 = 0, 1, 2, 3
(ARB_STAGE_QKV, ARB_STAGE_ATTENTION, ARB_STAGE_OPROJ, ARB_STAGE_GATE_UP, ARB_STAGE_DOWN, ARB_STAGE_NORM,
 ARB_STAGE_ROPE_APPEND, ARB_STAGE_GATE_UP_LARGE) = range(8)
_STATUS = {0: "ARB_OK", 1: "ARB_EINVAL", 2: "ARB_ESHAPE", 3: "ARB_ECAPACITY", 4: "ARB_EHIP", 5: "ARB_EUNSUPPORTED"}

NOALLOC_SCRATCH_BYTES = 64 << 20      # ARB_NOALLOC_SCRATCH_BYTES of include/arb.h

EXPORTS = ["arb_model_create", "arb_model_destroy", "arb_workspace_bytes", "arb_score_steps", "arb_score_steps_noalloc", "arb_prefill",
           "arb_route", "arb_next_token", "arb_next_token_workspace_bytes", "arb_first_stop", "arb_step_advance", "arb_pack_steps", "arb_advantage_route", "arb_budget_threshold", "arb_slot_mapping", "arb_stage_gemm", "arb_pack_k_blocked", "arb_w4_quantize", "arb_w3_quantize", "arb_stage_gemm_w4", "arb_stage_attention", "arb_stage_rmsnorm",
           "arb_stage_rope_append", "arb_stage_norm_pool_head", "arb_stage_layers", "arb_gemm_large_tile_columns", "arb_model_trace", "arb_model_trace_count",
           "arb_last_error"]


class ArbError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rms_eps", C.c_float), ("rope_base", C.c_float), ("kv_block", C.c_int32), ("pool", C.c_int32),
                ("has_router_head", C.c_int32)]


class _Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("wqkv", C.POINTER(C.c_void_p)), ("wo", C.POINTER(C.c_void_p)),
                ("wgu", C.POINTER(C.c_void_p)), ("wd", C.POINTER(C.c_void_p)), ("g_attn", C.POINTER(C.c_void_p)),
                ("g_mlp", C.POINTER(C.c_void_p)), ("g_final", C.c_void_p), ("w_head", C.c_void_p),
                ("b_head", C.c_float), ("wqkv_scale", C.POINTER(C.c_void_p)), ("wo_scale", C.POINTER(C.c_void_p)),
                ("wgu_scale", C.POINTER(C.c_void_p)), ("wd_scale", C.POINTER(C.c_void_p)),
                ("wgu_blocked", C.POINTER(C.c_void_p))]


class _KV(C.Structure):
    _fields_ = [("k_pool", C.POINTER(C.c_void_p)), ("v_pool", C.POINTER(C.c_void_p)), ("n_blocks", C.c_int32)]


class _Batch(C.Structure):
    _fields_ = [("batch", C.c_int32), ("total_tokens", C.c_int32), ("max_blocks_per_seq", C.c_int32),
                ("token_ids", C.c_void_p), ("block_tables", C.c_void_p), ("prefix_lens", C.c_void_p),
                ("cu_step_lens", C.c_void_p), ("prefix_lens_host", C.c_void_p), ("cu_step_lens_host", C.c_void_p)]


def load_library(path: Optional[str] = None):
    """Loads libarb.so (built in-tree by build.py).  Raises if it is not there."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or _LIB_PATH
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is not built; run `python -m paper_2512_05033_amd.build` "
                           "(there is no fallback implementation)")
    lib = C.CDLL(path)
    lib.arb_last_error.restype = C.c_char_p
    lib.arb_workspace_bytes.restype = C.c_size_t
    lib.arb_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32]
    lib.arb_model_create.argtypes = [C.POINTER(_Cfg), C.POINTER(_Weights), C.POINTER(C.c_void_p)]
    lib.arb_model_destroy.argtypes = [C.c_void_p]
    lib.arb_score_steps.argtypes = [C.c_void_p, C.POINTER(_KV), C.POINTER(_Batch), C.c_float, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.arb_score_steps_noalloc.argtypes = [C.c_void_p, C.POINTER(_KV), C.POINTER(_Batch), C.c_float, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_void_p]
    lib.arb_prefill.argtypes = [C.c_void_p, C.POINTER(_KV), C.POINTER(_Batch), C.c_void_p, C.c_void_p, C.c_size_t,
                                C.c_void_p]
    lib.arb_route.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_int32, C.c_void_p, C.c_void_p]
    lib.arb_advantage_route.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p]
    lib.arb_budget_threshold.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.arb_next_token_workspace_bytes.argtypes = [C.c_int32] * 3
    lib.arb_next_token_workspace_bytes.restype = C.c_size_t
    lib.arb_next_token.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_float,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.arb_first_stop.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                   C.c_void_p]
    lib.arb_step_advance.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.arb_pack_steps.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    lib.arb_slot_mapping.argtypes = [C.POINTER(_Batch), C.c_int32, C.c_void_p, C.c_void_p]
    lib.arb_stage_gemm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                   C.c_int32, C.c_void_p]
    lib.arb_w4_quantize.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.arb_w3_quantize.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.arb_pack_k_blocked.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p]
    lib.arb_stage_gemm_w4.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                      C.c_int32, C.c_void_p]
    lib.arb_stage_attention.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                        C.POINTER(_Batch), C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.arb_stage_rmsnorm.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.arb_stage_rope_append.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(_Batch),
                                          C.c_void_p, C.c_size_t, C.c_void_p]
    lib.arb_stage_norm_pool_head.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.POINTER(_Batch), C.c_int32,
                                             C.c_void_p, C.c_float, C.c_int32, C.c_float, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.arb_stage_layers.argtypes = [C.c_void_p, C.POINTER(_KV), C.POINTER(_Batch), C.c_int32, C.c_int32, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.arb_model_trace.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int32]
    lib.arb_model_trace_count.argtypes = [C.c_void_p]
    lib.arb_model_trace_count.restype = C.c_int32
    lib.arb_gemm_large_tile_columns.argtypes = [C.c_int32] * 4
    lib.arb_gemm_large_tile_columns.restype = C.c_int32
    for name in EXPORTS:
        if name not in ("arb_last_error", "arb_workspace_bytes", "arb_model_trace_count", "arb_gemm_large_tile_columns",
                        "arb_next_token_workspace_bytes"):
            getattr(lib, name).restype = C.c_int
    if path == _LIB_PATH:
        _lib = lib
    return lib


def _check(status: int):
    if status != ARB_OK:
        raise ArbError(status, load_library().arb_last_error().decode())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _ptr_array(tensors: Sequence[torch.Tensor]):
    return (C.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])


def _dev(t: torch.Tensor, dtype) -> torch.Tensor:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"expected a contiguous cuda tensor of {dtype}, got {t.dtype} on {t.device}")
    return t


class Model:
    """An arb_model plus the tensors it points at (kept alive here)."""

    def __init__(self, *, n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, weights,
                 rms_eps=1e-6, rope_base=10000.0, kv_block=16, pool=ARB_POOL_MEAN, has_router_head=True,
                 block_gate_up=True):
        """block_gate_up: also hand the library K-blocked copies of the gate/up weights (arb_pack_k_blocked; made
        here on the weights' device, 4 F d bytes per layer); bf16 weights only."""
        lib = load_library()
        w = weights
        bf, f32 = torch.bfloat16, torch.float32
        scales = getattr(w, "scales", None)                   # set: 4-bit projection weights (QuantizedWeights)
        proj = torch.int32 if scales is not None else bf
        self._keep = [_dev(w.embed, bf), *[_dev(t, proj) for l in (w.wqkv, w.wo, w.wgu, w.wd) for t in l],
                      *[_dev(t, f32) for l in (w.g_attn, w.g_mlp) for t in l], _dev(w.g_final, f32)]
        head_kind = ARB_HEAD_NONE
        if has_router_head:
            self._keep.append(_dev(w.w_head, f32))
            # a [2, d] head is the two-class head (scores are class-1 probabilities), a [d] head the linear one
            head_kind = ARB_HEAD_TWO_CLASS if w.w_head.dim() == 2 else ARB_HEAD_LINEAR
            if tuple(w.w_head.shape) not in ((d_model,), (2, d_model)):
                raise ValueError(f"w_head has shape {tuple(w.w_head.shape)}")
        self.cfg = _Cfg(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, rms_eps, rope_base,
                        kv_block, pool, head_kind)
        self._arrays = [_ptr_array(l) for l in (w.wqkv, w.wo, w.wgu, w.wd, w.g_attn, w.g_mlp)]
        self._scale_arrays = [None] * 4
        if scales is not None:
            self._keep += [_dev(t, bf) for l in scales for t in l]
            self._scale_arrays = [_ptr_array(l) for l in scales]
        blocked = None
        if block_gate_up and scales is None and w.wgu[0].is_cuda and d_model % 32 == 0:
            self._keep += (packed := [arb_pack_k_blocked(t) for t in w.wgu])
            torch.cuda.synchronize(w.embed.device)  # packed on torch's stream; callers may use any other
            blocked = _ptr_array(packed)
            self._arrays.append(blocked)           # keeps the pointer table alive
        cw = _Weights(w.embed.data_ptr(), *self._arrays[:6], w.g_final.data_ptr(),
                      w.w_head.data_ptr() if has_router_head else None, float(w.b_head), *self._scale_arrays, blocked)
        self.handle = C.c_void_p()
        _check(lib.arb_model_create(C.byref(self.cfg), C.byref(cw), C.byref(self.handle)))
        self.weights = w
        self.device = w.embed.device

    def workspace_bytes(self, max_batch: int, max_total_tokens: int, max_ctx: int) -> int:
        return int(load_library().arb_workspace_bytes(self.handle, max_batch, max_total_tokens, max_ctx))

    def close(self):
        if getattr(self, "handle", None):
            load_library().arb_model_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class KVCache:
    """Per-layer K and V pools, bf16 [n_blocks, Hkv, kv_block, head_dim] on the device."""

    def __init__(self, k_pools: List[torch.Tensor], v_pools: List[torch.Tensor]):
        self.k_pools = [_dev(t, torch.bfloat16) for t in k_pools]
        self.v_pools = [_dev(t, torch.bfloat16) for t in v_pools]
        self._k, self._v = _ptr_array(self.k_pools), _ptr_array(self.v_pools)
        self.c = _KV(self._k, self._v, int(k_pools[0].shape[0]))


class DeviceBatch:
    """Lengths on host and device, block tables and token ids on the device."""

    def __init__(self, prefix_lens, cu_step_lens, block_tables, token_ids=None, device="cuda"):
        self.prefix_host = np.ascontiguousarray(prefix_lens, dtype=np.int32)
        self.cu_host = np.ascontiguousarray(cu_step_lens, dtype=np.int32)
        tables = np.ascontiguousarray(block_tables, dtype=np.int32)
        to = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(device)
        self.prefix, self.cu, self.tables = to(self.prefix_host), to(self.cu_host), to(tables)
        if isinstance(token_ids, torch.Tensor):           # already on the device (tokens chosen by arb_next_token)
            self.tokens = _dev(token_ids, torch.int32)
        else:
            self.tokens = None if token_ids is None else to(token_ids)
        self.batch = len(self.prefix_host)
        self.total_tokens = int(self.cu_host[-1]) if len(self.cu_host) else 0
        self.c = _Batch(self.batch, self.total_tokens, tables.shape[1] if tables.ndim == 2 else 0,
                        _ptr(self.tokens), _ptr(self.tables), _ptr(self.prefix), _ptr(self.cu),
                        self.prefix_host.ctypes.data, self.cu_host.ctypes.data)

    @property
    def max_ctx(self) -> int:
        return int((self.prefix_host + np.diff(self.cu_host)).max()) if self.batch else 0


def _workspace(model: Model, batch: DeviceBatch, ws: Optional[torch.Tensor]) -> torch.Tensor:
    if ws is None:
        n = model.workspace_bytes(batch.batch, batch.total_tokens, batch.max_ctx)
        ws = torch.empty(max(n, 256), dtype=torch.uint8, device=model.device)
    return ws


def arb_score_steps(model: Model, kv: KVCache, batch: DeviceBatch, tau: float, *, want_hidden: bool = False,
                    ws: Optional[torch.Tensor] = None, scores=None, escalate=None, hidden=None, stream=None):
    """-> (scores fp32 [B] or None, escalate uint8 [B] or None, hidden bf16 [T, d] or None)."""
    head = bool(model.cfg.has_router_head)
    dev = model.device
    if head and scores is None:
        scores = torch.empty(batch.batch, dtype=torch.float32, device=dev)
    if head and escalate is None:
        escalate = torch.empty(batch.batch, dtype=torch.uint8, device=dev)
    if want_hidden and hidden is None:
        hidden = torch.empty(batch.total_tokens, model.cfg.d_model, dtype=torch.bfloat16, device=dev)
    ws = _workspace(model, batch, ws)
    _check(load_library().arb_score_steps(model.handle, C.byref(kv.c), C.byref(batch.c), float(tau), _ptr(scores),
                                          _ptr(escalate), _ptr(hidden), ws.data_ptr(), ws.numel(), _stream(stream)))
    return scores, escalate, hidden


def arb_score_steps_noalloc(model: Model, kv: KVCache, batch: DeviceBatch, tau: float, *, scores=None, escalate=None,
                            hidden=None, stream=None):
    """arb_score_steps on the library's static scratch buffer.  The caller passes every output tensor
    (scores and escalate when the model has a head; hidden optional); nothing is allocated here."""
    _check(load_library().arb_score_steps_noalloc(model.handle, C.byref(kv.c), C.byref(batch.c), float(tau),
                                                  _ptr(scores), _ptr(escalate), _ptr(hidden), _stream(stream)))
    return scores, escalate, hidden


def arb_prefill(model: Model, kv: KVCache, batch: DeviceBatch, *, want_hidden: bool = False,
                ws: Optional[torch.Tensor] = None, stream=None):
    hidden = None
    if want_hidden:
        hidden = torch.empty(batch.total_tokens, model.cfg.d_model, dtype=torch.bfloat16, device=model.device)
    ws = _workspace(model, batch, ws)
    _check(load_library().arb_prefill(model.handle, C.byref(kv.c), C.byref(batch.c), _ptr(hidden), ws.data_ptr(),
                                      ws.numel(), _stream(stream)))
    return hidden


def arb_route(scores: torch.Tensor, tau: float, sense: int = ARB_ESCALATE_IF_GT, stream=None) -> torch.Tensor:
    _dev(scores, torch.float32)
    out = torch.empty(scores.numel(), dtype=torch.uint8, device=scores.device)
    _check(load_library().arb_route(_ptr(scores), scores.numel(), float(tau), sense, _ptr(out), _stream(stream)))
    return out


def arb_advantage_route(s_t: torch.Tensor, s_d: torch.Tensor, tau=0.0, stream=None):
    """-> (delta fp32 [n], escalate uint8 [n], realized fp32 [n]); tau: a float, or a 1-element device tensor."""
    _dev(s_t, torch.float32), _dev(s_d, torch.float32)
    n = s_t.numel()
    if s_d.numel() != n:
        raise ValueError("score arrays differ in length")
    delta, realized = torch.empty_like(s_t), torch.empty_like(s_t)
    esc = torch.empty(n, dtype=torch.uint8, device=s_t.device)
    tau_dev = _dev(tau, torch.float32) if isinstance(tau, torch.Tensor) else None
    _check(load_library().arb_advantage_route(_ptr(s_t), _ptr(s_d), n, 0.0 if tau_dev is not None else float(tau),
                                           _ptr(tau_dev), _ptr(delta), _ptr(esc), _ptr(realized), _stream(stream)))
    return delta, esc, realized


def arb_budget_threshold(delta: torch.Tensor, budget: int, stream=None) -> torch.Tensor:
    """-> 1-element device tensor holding tau (Theorem B.1)."""
    _dev(delta, torch.float32)
    out = torch.empty(1, dtype=torch.float32, device=delta.device)
    _check(load_library().arb_budget_threshold(_ptr(delta), delta.numel(), int(budget), _ptr(out), _stream(stream)))
    return out


def arb_next_token(hidden: torch.Tensor, rows: torch.Tensor, w_lm: torch.Tensor, temperature: float = 0.0,
                   uniforms: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None, stream=None):
    """-> (token int32 [n], chosen logit fp32 [n]) for the hidden rows `rows` (int32 device tensor)."""
    _dev(hidden, torch.bfloat16), _dev(rows, torch.int32), _dev(w_lm, torch.bfloat16)
    n, d, V = rows.numel(), hidden.shape[1], w_lm.shape[0]
    if w_lm.shape[1] != d:
        raise ValueError("LM head width")
    if uniforms is not None:
        _dev(uniforms, torch.float32)
    lib = load_library()
    need = int(lib.arb_next_token_workspace_bytes(n, d, V))
    if ws is None:
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device=hidden.device)
    token = torch.empty(n, dtype=torch.int32, device=hidden.device)
    chosen = torch.empty(n, dtype=torch.float32, device=hidden.device)
    _check(lib.arb_next_token(_ptr(hidden), _ptr(rows), n, d, _ptr(w_lm), V, float(temperature), _ptr(uniforms),
                              _ptr(token), _ptr(chosen), ws.data_ptr(), ws.numel(), _stream(stream)))
    return token, chosen


def arb_first_stop(tokens: torch.Tensor, sep: int, eos: int, stream=None):
    """tokens int32 [n, max_len] -> (len int32 [n], ended uint8 [n])."""
    _dev(tokens, torch.int32)
    n, S = tokens.shape
    length = torch.empty(n, dtype=torch.int32, device=tokens.device)
    ended = torch.empty(n, dtype=torch.uint8, device=tokens.device)
    _check(load_library().arb_first_stop(_ptr(tokens), n, S, int(sep), int(eos), _ptr(length), _ptr(ended),
                                         _stream(stream)))
    return length, ended


def arb_step_advance(open_rows: torch.Tensor, chosen: torch.Tensor, steps: torch.Tensor, length: torch.Tensor,
                     done: torch.Tensor, sep: int, eos: int, next_buf: torch.Tensor, next_ids: torch.Tensor, stream=None):
    """One decoding iteration: appends chosen[j] to row open_rows[j] of steps (int32 [n, max_len]; length int32 [n],
    done uint8 [n] updated in place).  next_buf int32 [1 + n_open]: element 0 receives the number of rows that stay
    open, the elements behind it those rows; next_ids int32 [n_open] receives their tokens."""
    for t in (open_rows, chosen, steps, length, next_buf, next_ids):
        _dev(t, torch.int32)
    _dev(done, torch.uint8)
    n, S = steps.shape
    n_open = open_rows.numel()
    if chosen.numel() != n_open or next_buf.numel() < 1 + n_open or next_ids.numel() < n_open:
        raise ValueError("arb_step_advance: buffer sizes")
    _check(load_library().arb_step_advance(_ptr(open_rows), _ptr(chosen), n_open, n, S, int(sep), int(eos), _ptr(steps),
                                           _ptr(length), _ptr(done), next_buf.data_ptr() + 4, _ptr(next_ids),
                                           next_buf.data_ptr(), _stream(stream)))


def arb_pack_steps(steps: torch.Tensor, rows: torch.Tensor, cu: torch.Tensor, total: int, stream=None) -> torch.Tensor:
    """-> ids int32 [total]: the steps of `rows` (tokens steps[r][: cu[j+1] - cu[j]]) one after the other."""
    for t in (steps, rows, cu):
        _dev(t, torch.int32)
    ids = torch.empty(total, dtype=torch.int32, device=steps.device)
    _check(load_library().arb_pack_steps(_ptr(steps), steps.shape[1], _ptr(rows), _ptr(cu), rows.numel(), _ptr(ids),
                                         _stream(stream)))
    return ids


def arb_slot_mapping(batch: DeviceBatch, kv_block: int = 16, stream=None) -> torch.Tensor:
    out = torch.empty(batch.total_tokens, dtype=torch.int32, device=batch.tables.device)
    _check(load_library().arb_slot_mapping(C.byref(batch.c), kv_block, _ptr(out), _stream(stream)))
    return out


def arb_stage_gemm(a: torch.Tensor, b: torch.Tensor, epilogue: int = ARB_EPI_STORE_BF16,
                   out: Optional[torch.Tensor] = None, stream=None, b_blocked: Optional[torch.Tensor] = None) -> torch.Tensor:
    """a bf16 [M, K], b bf16 [N, K] (or [2F, K] for SwiGLU) -> [M, N] (or [M, F]); b_blocked: arb_pack_k_blocked(b)."""
    _dev(a, torch.bfloat16), _dev(b, torch.bfloat16)
    if b_blocked is not None and (_dev(b_blocked, torch.bfloat16).numel() != b.numel() or a.shape[1] % 32):
        raise ValueError("b_blocked does not match b")
    M, K = a.shape
    N = b.shape[0] // 2 if epilogue == ARB_EPI_SWIGLU_BF16 else b.shape[0]
    if b.shape[1] != K:
        raise ValueError("inner dimensions differ")
    if out is None:
        if epilogue == ARB_EPI_RESIDUAL_F32:
            raise ValueError("the residual epilogue accumulates into `out`")
        out = torch.empty(M, N, dtype=torch.float32 if epilogue == ARB_EPI_STORE_F32 else torch.bfloat16, device=a.device)
    _dev(out, torch.float32 if epilogue in (ARB_EPI_RESIDUAL_F32, ARB_EPI_STORE_F32) else torch.bfloat16)
    if tuple(out.shape) != (M, N):
        raise ValueError("output shape")
    _check(load_library().arb_stage_gemm(_ptr(a), _ptr(b), _ptr(b_blocked) if b_blocked is not None else None,
                                         _ptr(out), M, N, K, epilogue, _stream(stream)))
    return out


def arb_pack_k_blocked(w: torch.Tensor, stream=None) -> torch.Tensor:
    """bf16 [rows, K] -> its K-blocked copy, bf16 [K/32, rows, 32]."""
    _dev(w, torch.bfloat16)
    rows, K = w.shape
    if K % 32:
        raise ValueError("K must be a multiple of 32")
    packed = torch.empty(K // 32, rows, 32, dtype=torch.bfloat16, device=w.device)
    _check(load_library().arb_pack_k_blocked(_ptr(w), rows, K, _ptr(packed), _stream(stream)))
    return packed


def _quantize(entry, w: torch.Tensor, stream):
    _dev(w, torch.bfloat16)
    N, K = w.shape
    if K % 128:
        raise ValueError("K must be a multiple of 128")
    packed = torch.empty(N, K // 8, dtype=torch.int32, device=w.device)
    scales = torch.empty(N, K // 128, dtype=torch.bfloat16, device=w.device)
    _check(getattr(load_library(), entry)(_ptr(w), N, K, _ptr(packed), _ptr(scales), _stream(stream)))
    return packed, scales


def arb_w4_quantize(w: torch.Tensor, stream=None):
    """bf16 [N, K] -> (packed int32 [N, K/8] (the uint32 words), scales bf16 [N, K/128])."""
    return _quantize("arb_w4_quantize", w, stream)


def arb_w3_quantize(w: torch.Tensor, stream=None):
    """The same with 3-bit integers (-4..3) in the same nibble format."""
    return _quantize("arb_w3_quantize", w, stream)


def arb_stage_gemm_w4(a: torch.Tensor, packed: torch.Tensor, scales: torch.Tensor, epilogue: int = ARB_EPI_STORE_BF16,
                      out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """a bf16 [M, K], 4-bit weights of arb_w4_quantize for [N, K] (or [2F, K] for SwiGLU) -> [M, N] (or [M, F])."""
    _dev(a, torch.bfloat16), _dev(packed, torch.int32), _dev(scales, torch.bfloat16)
    M, K = a.shape
    rows = packed.shape[0]
    N = rows // 2 if epilogue == ARB_EPI_SWIGLU_BF16 else rows
    if packed.shape[1] * 8 != K or tuple(scales.shape) != (rows, K // 128):
        raise ValueError("weight shapes")
    f32_out = epilogue in (ARB_EPI_RESIDUAL_F32, ARB_EPI_STORE_F32)
    if out is None:
        if epilogue == ARB_EPI_RESIDUAL_F32:
            raise ValueError("the residual epilogue accumulates into `out`")
        out = torch.empty(M, N, dtype=torch.float32 if f32_out else torch.bfloat16, device=a.device)
    _dev(out, torch.float32 if f32_out else torch.bfloat16)
    _check(load_library().arb_stage_gemm_w4(_ptr(a), _ptr(packed), _ptr(scales), _ptr(out), M, N, K, epilogue,
                                            _stream(stream)))
    return out


class QuantizedWeights:
    """The weights of a model with its four projection matrices per layer in the 4-bit format (bits = 3: 3-bit integers in it)."""

    def __init__(self, w, bits: int = 4):
        self.embed, self.g_attn, self.g_mlp, self.g_final = w.embed, w.g_attn, w.g_mlp, w.g_final
        self.w_head, self.b_head = w.w_head, w.b_head
        quantize = {4: arb_w4_quantize, 3: arb_w3_quantize}[bits]
        pairs = [[quantize(t) for t in l] for l in (w.wqkv, w.wo, w.wgu, w.wd)]
        self.wqkv, self.wo, self.wgu, self.wd = ([p for p, _ in l] for l in pairs)
        self.scales = [[s for _, s in l] for l in pairs]


def arb_gemm_large_tile_columns(M: int, N: int, K: int, epilogue: int) -> int:
    return int(load_library().arb_gemm_large_tile_columns(M, N, K, epilogue))


def arb_stage_attention(model: Model, q: torch.Tensor, k_pool: torch.Tensor, v_pool: torch.Tensor,
                        batch: DeviceBatch, ws: Optional[torch.Tensor] = None, stream=None,
                        q_scaled: bool = False) -> torch.Tensor:
    """q bf16 [T, row] whose first Hq*hd columns are the (rotated) query heads -> bf16 [T, Hq*hd].
    q_scaled: q already carries the factor log2(e)/sqrt(head_dim)."""
    _dev(q, torch.bfloat16), _dev(k_pool, torch.bfloat16), _dev(v_pool, torch.bfloat16)
    out = torch.empty(batch.total_tokens, model.cfg.n_q_heads * model.cfg.head_dim, dtype=torch.bfloat16,
                      device=q.device)
    ws = _workspace(model, batch, ws)
    _check(load_library().arb_stage_attention(model.handle, _ptr(q), q.shape[1], int(q_scaled), _ptr(k_pool), _ptr(v_pool),
                                              C.byref(batch.c), _ptr(out), ws.data_ptr(), ws.numel(), _stream(stream)))
    return out


def arb_stage_rmsnorm(x: torch.Tensor, g: torch.Tensor, eps: float, stream=None) -> torch.Tensor:
    _dev(x, torch.float32), _dev(g, torch.float32)
    out = torch.empty(x.shape, dtype=torch.bfloat16, device=x.device)
    _check(load_library().arb_stage_rmsnorm(_ptr(x), _ptr(g), float(eps), x.shape[0], x.shape[1], _ptr(out),
                                            _stream(stream)))
    return out


def arb_stage_rope_append(model: Model, qkv: torch.Tensor, k_pool: torch.Tensor, v_pool: torch.Tensor,
                          batch: DeviceBatch, stream=None) -> None:
    """Rotates the q heads of qkv in place and appends rotated k and v to the pool."""
    _dev(qkv, torch.bfloat16), _dev(k_pool, torch.bfloat16), _dev(v_pool, torch.bfloat16)
    ws = _workspace(model, batch, None)
    _check(load_library().arb_stage_rope_append(model.handle, _ptr(qkv), _ptr(k_pool), _ptr(v_pool), C.byref(batch.c),
                                                ws.data_ptr(), ws.numel(), _stream(stream)))


def arb_stage_norm_pool_head(h: torch.Tensor, g_final: torch.Tensor, eps: float, batch: DeviceBatch,
                             w_head: torch.Tensor, b_head: float, pool: int, tau: float, want_hidden=True, stream=None):
    _dev(h, torch.float32), _dev(g_final, torch.float32), _dev(w_head, torch.float32)
    T, d = h.shape
    hidden = torch.empty(T, d, dtype=torch.bfloat16, device=h.device) if want_hidden else None
    scores = torch.empty(batch.batch, dtype=torch.float32, device=h.device)
    esc = torch.empty(batch.batch, dtype=torch.uint8, device=h.device)
    ws = torch.empty(max(4 * T, 256), dtype=torch.uint8, device=h.device)
    _check(load_library().arb_stage_norm_pool_head(_ptr(h), _ptr(g_final), float(eps), C.byref(batch.c), d,
                                                   _ptr(w_head), float(b_head), pool, float(tau), _ptr(hidden),
                                                   _ptr(scores), _ptr(esc), ws.data_ptr(), ws.numel(), _stream(stream)))
    return scores, esc, hidden


def arb_stage_layers(model: Model, kv: KVCache, batch: DeviceBatch, layer_begin: int, layer_end: int,
                     h_in: torch.Tensor, ws: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """h_in fp32 [T, d], the residual stream entering layer_begin -> the stream leaving layer_end - 1."""
    _dev(h_in, torch.float32)
    if tuple(h_in.shape) != (batch.total_tokens, model.cfg.d_model):
        raise ValueError("residual stream shape")
    h_out = torch.empty_like(h_in)
    ws = _workspace(model, batch, ws)
    _check(load_library().arb_stage_layers(model.handle, C.byref(kv.c), C.byref(batch.c), layer_begin, layer_end,
                                           _ptr(h_in), _ptr(h_out), ws.data_ptr(), ws.numel(), _stream(stream)))
    return h_out


class StageTimer:
    """HIP events the library records around every launch of one stage of the
    forward (arb_model_trace), on the stream the kernels run on."""

    def __init__(self, model: Model, stage: int, capacity: int):
        self.model, self.stage, self.n = model, stage, capacity
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]
        self.start, self.stop = (C.c_void_p * capacity)(), (C.c_void_p * capacity)()
        for arr in (self.start, self.stop):
            for i in range(capacity):
                ev = C.c_void_p()
                if self.hip.hipEventCreate(C.byref(ev)) != 0:
                    raise RuntimeError("hipEventCreate failed")
                arr[i] = ev

    def arm(self):
        _check(load_library().arb_model_trace(self.model.handle, self.stage, self.start, self.stop, self.n))

    def disarm(self):
        count = load_library().arb_model_trace_count(self.model.handle)
        _check(load_library().arb_model_trace(self.model.handle, self.stage, None, None, 0))
        return count

    def durations_ms(self, count: int):
        """Per-launch durations; call after the stream has been synchronised."""
        out = []
        for i in range(count):
            ms = C.c_float()
            if self.hip.hipEventElapsedTime(C.byref(ms), self.start[i], self.stop[i]) != 0:
                raise RuntimeError("hipEventElapsedTime failed")
            out.append(ms.value)
        return out

    def close(self):
        for arr in (self.start, self.stop):
            for i in range(self.n):
                if arr[i]:
                    self.hip.hipEventDestroy(arr[i])
                    arr[i] = None
