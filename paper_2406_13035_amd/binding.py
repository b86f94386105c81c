"""Thin ctypes binding of libd2o.so: argument marshalling only, same names as include/d2o.h.

PyTorch is used for device memory (workspaces, tensors) and the current stream; every step
of the path runs in the library's HIP kernels.  There is no CPU fallback: if the library is
missing or a call fails, an exception is raised."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("D2O_LIB", os.path.join(HERE, "libd2o.so"))

D2O_F32, D2O_BF16 = 0, 1
EXPORTS = [
    "d2o_workspace_bytes", "d2o_qkv_project", "d2o_create", "d2o_destroy", "d2o_last_error", "d2o_reset",
    "d2o_prefill_attend", "d2o_get_density", "d2o_allocate_budgets", "d2o_allocate_budgets_policy",
    "d2o_scores_import",
    "d2o_scores_export", "d2o_compress_layer", "d2o_compress_layer_heads", "d2o_allocate_budgets_heads", "d2o_candidate_misses", "d2o_prefill_compress", "d2o_decode_step",
    "d2o_decode_step_static", "d2o_append_chunk", "d2o_append_events",
    "d2o_layer_reserve", "d2o_cache_export", "d2o_cache_import", "d2o_last_events",
    "d2o_prefill_events", "d2o_timing_enable", "d2o_timing_read",
]


class D2OError(RuntimeError):
    pass


class d2o_config(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_layers", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("max_prompt_len", C.c_int32),
                ("slots_per_seq", C.c_int64), ("dtype", C.c_int32), ("n_sink", C.c_int32),
                ("beta", C.c_double), ("tau_force", C.c_double), ("out_f32", C.c_int32),
                ("merge_average", C.c_int32), ("max_append", C.c_int32),
                ("split_rows", C.c_int32), ("cache_fp8", C.c_int32)]


class d2o_view(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("stride_b", C.c_int64), ("stride_h", C.c_int64),
                ("stride_n", C.c_int64)]


_lib = None


def load_library() -> C.CDLL:
    """Loads the built library; builds nothing.  Raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise D2OError(f"{LIB_PATH} not found: run `python -m paper_2406_13035_amd.build` "
                       "(or __graft_entry__.build()) first; there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    P = C.POINTER
    lib.d2o_workspace_bytes.argtypes = [P(d2o_config), P(C.c_size_t), P(C.c_size_t)]
    lib.d2o_qkv_project.argtypes = [i32, i32, i32, i32, i32, i32, i32, vp, vp, d2o_view, d2o_view, d2o_view, i32,
                                    C.c_double, vp]
    lib.d2o_create.argtypes = [P(d2o_config), vp, C.c_size_t, vp, C.c_size_t, vp, P(vp)]
    lib.d2o_destroy.argtypes = [vp]
    lib.d2o_destroy.restype = None
    lib.d2o_last_error.argtypes = [vp]
    lib.d2o_last_error.restype = C.c_char_p
    lib.d2o_reset.argtypes = [vp, vp]
    lib.d2o_prefill_attend.argtypes = [vp, i32, d2o_view, d2o_view, d2o_view, i32, d2o_view, vp]
    lib.d2o_get_density.argtypes = [vp, vp, vp, vp]
    lib.d2o_allocate_budgets.argtypes = [vp, i32, i32, i64, i32, vp]
    lib.d2o_allocate_budgets_policy.argtypes = [i32, vp, i32, i32, i64, i32, vp]
    lib.d2o_scores_import.argtypes = [vp, i32, vp, i32, vp]
    lib.d2o_scores_export.argtypes = [vp, i32, vp, i32, vp]
    lib.d2o_compress_layer.argtypes = [vp, i32, d2o_view, d2o_view, i32, vp, vp, vp]
    lib.d2o_compress_layer_heads.argtypes = [vp, i32, d2o_view, d2o_view, i32, vp, vp, vp]
    lib.d2o_allocate_budgets_heads.argtypes = [vp, i32, i32, i32, i32, i64, i32, vp]
    lib.d2o_prefill_compress.argtypes = [vp, i32, d2o_view, d2o_view, d2o_view, i32, d2o_view,
                                         vp, vp, vp]
    lib.d2o_decode_step.argtypes = [vp, i32, i32, d2o_view, d2o_view, d2o_view, d2o_view, vp]
    lib.d2o_decode_step_static.argtypes = [vp, i32, i32, d2o_view, d2o_view, d2o_view, d2o_view, vp]
    lib.d2o_append_chunk.argtypes = [vp, i32, d2o_view, d2o_view, d2o_view, i32, d2o_view, vp]
    lib.d2o_append_events.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.d2o_layer_reserve.argtypes = [vp, i32, i32, vp, vp]
    lib.d2o_cache_export.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.d2o_cache_import.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, i32, C.c_double, i32, vp]
    lib.d2o_last_events.argtypes = [vp, i32, vp, vp, vp, vp]
    lib.d2o_prefill_events.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.d2o_timing_enable.argtypes = [vp, i32]
    lib.d2o_timing_read.argtypes = [vp, i32, P(C.c_double), P(C.c_int64), vp]
    for name in EXPORTS:
        if name not in ("d2o_destroy", "d2o_last_error"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _np_ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def d2o_allocate_budgets(F, seq_len: int, total_budget: int, min_budget: int = 64) -> np.ndarray:
    """Sec. 4.1 Eq. 5: integer layer budgets from the density statistics (host function)."""
    lib = load_library()
    F = np.ascontiguousarray(F, dtype=np.float64)
    S = np.zeros(F.size, dtype=np.int32)
    rc = lib.d2o_allocate_budgets(_np_ptr(F), F.size, seq_len, total_budget, min_budget, _np_ptr(S))
    if rc != 0:
        raise D2OError(f"d2o_allocate_budgets failed with {rc}")
    return S


def d2o_allocate_budgets_heads(F_heads, n_kv_heads: int, seq_len: int, total_budget: int,
                               min_budget: int = 64) -> np.ndarray:
    """App. A.8: per-(layer, KV head) budgets from the per-query-head variances [L][Hq] (host function)."""
    lib = load_library()
    F = np.ascontiguousarray(F_heads, dtype=np.float64)
    L, Hq = F.shape
    S = np.zeros((L, n_kv_heads), dtype=np.int32)
    rc = lib.d2o_allocate_budgets_heads(_np_ptr(F), L, Hq, n_kv_heads, seq_len, total_budget, min_budget, _np_ptr(S))
    if rc != 0:
        raise D2OError(f"d2o_allocate_budgets_heads failed with {rc}")
    return S


def d2o_qkv_project(X: torch.Tensor, W: torch.Tensor, n_q_heads: int, n_kv_heads: int, head_dim: int,
                    pos0: int = 0, rope_base: float = 10000.0):
    """Sec. 3 Eq. 1 with rotary embedding: X [B, n, hidden], W [(Hq + 2 Hkv) d, hidden] (bf16, on the
    device) -> Q [B, Hq, n, d], K, V [B, Hkv, n, d]."""
    lib = load_library()
    assert X.is_cuda and W.is_cuda and X.dtype == torch.bfloat16 and W.dtype == torch.bfloat16
    assert X.is_contiguous() and W.is_contiguous()
    B, n, hidden = X.shape
    Q = torch.empty((B, n_q_heads, n, head_dim), dtype=X.dtype, device=X.device)
    K = torch.empty((B, n_kv_heads, n, head_dim), dtype=X.dtype, device=X.device)
    V = torch.empty_like(K)
    with torch.cuda.device(X.device):
        rc = lib.d2o_qkv_project(B, n, hidden, n_q_heads, n_kv_heads, head_dim, D2O_BF16, X.data_ptr(), W.data_ptr(),
                                 view4(Q), view4(K), view4(V), pos0, rope_base, _stream_ptr())
    if rc != 0:
        raise D2OError(f"d2o_qkv_project failed with {rc}")
    return Q, K, V


ALLOC_POLICIES = {"softmax": 0, "reciprocal": 1, "exp_decay": 2, "uniform": 3}


def d2o_allocate_budgets_policy(policy: str, F, seq_len: int, total_budget: int, min_budget: int = 64) -> np.ndarray:
    """Layer budgets under one of the designs of alpha_l compared in Sec. 5 (host function)."""
    lib = load_library()
    F = np.ascontiguousarray(F, dtype=np.float64)
    S = np.zeros(F.size, dtype=np.int32)
    rc = lib.d2o_allocate_budgets_policy(ALLOC_POLICIES[policy], _np_ptr(F), F.size, seq_len, total_budget,
                                         min_budget, _np_ptr(S))
    if rc != 0:
        raise D2OError(f"d2o_allocate_budgets_policy failed with {rc}")
    return S


def _stream_ptr() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def view4(t: torch.Tensor) -> d2o_view:
    """[b][head][token][d] tensor (any strides, d contiguous) as a d2o_view."""
    assert t.dim() == 4 and t.stride(3) == 1 and t.is_cuda
    return d2o_view(t.data_ptr(), t.stride(0), t.stride(1), t.stride(2))


def view_decode(t: torch.Tensor) -> d2o_view:
    """[layers][b][head][d] tensor as a d2o_view (stride_n = layer stride)."""
    assert t.dim() == 4 and t.stride(3) == 1 and t.is_cuda
    return d2o_view(t.data_ptr(), t.stride(1), t.stride(2), t.stride(0))


_NULL_VIEW = d2o_view(None, 0, 0, 0)


class D2O:
    """One library context plus the two device workspaces it lives in."""

    def __init__(self, batch, n_layers, n_q_heads, n_kv_heads, head_dim, max_prompt_len,
                 slots_per_seq, dtype="bf16", n_sink=0, beta=0.7, tau_force=float("nan"),
                 out_f32=False, device="cuda:0", merge_average=False, max_append=0, split_rows=0,
                 cache_fp8=False):
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise D2OError("no GPU visible: the D2O library has no CPU path")
        self.device = torch.device(device)
        self.cfg = d2o_config(batch, n_layers, n_q_heads, n_kv_heads, head_dim, max_prompt_len,
                              slots_per_seq, D2O_BF16 if dtype == "bf16" else D2O_F32, n_sink,
                              beta, tau_force, 1 if out_f32 else 0, 1 if merge_average else 0,
                              int(max_append), int(split_rows), 1 if cache_fp8 else 0)
        self.dtype = dtype
        self.out_dtype = torch.float32 if out_f32 else (torch.bfloat16 if dtype == "bf16" else torch.float32)
        self.torch_dtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.np_elem = np.uint16 if dtype == "bf16" else np.float32
        p, s = C.c_size_t(), C.c_size_t()
        rc = self.lib.d2o_workspace_bytes(C.byref(self.cfg), C.byref(p), C.byref(s))
        if rc != 0:
            raise D2OError(f"d2o_workspace_bytes failed with {rc}")
        self.persistent = torch.empty(p.value + 256, dtype=torch.uint8, device=self.device)
        self.scratch = torch.empty(s.value + 256, dtype=torch.uint8, device=self.device)
        pa = (self.persistent.data_ptr() + 255) & ~255
        sa = (self.scratch.data_ptr() + 255) & ~255
        ctx = C.c_void_p()
        with torch.cuda.device(self.device):
            rc = self.lib.d2o_create(C.byref(self.cfg), pa, p.value, sa, s.value, _stream_ptr(),
                                     C.byref(ctx))
        if rc != 0:
            raise D2OError(f"d2o_create failed with {rc}")
        self.ctx = ctx

    def close(self):
        if getattr(self, "ctx", None):
            self.lib.d2o_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc, what):
        if rc != 0:
            msg = self.lib.d2o_last_error(self.ctx)
            raise D2OError(f"{what} failed with {rc}: {msg.decode() if msg else ''}")

    # ---- calls, named as in d2o.h -------------------------------------------------------
    def d2o_reset(self):
        self._check(self.lib.d2o_reset(self.ctx, _stream_ptr()), "d2o_reset")

    def d2o_prefill_attend(self, layer, Q, K, V, O=None):
        n = Q.shape[2]
        ov = view4(O) if O is not None else _NULL_VIEW
        self._check(self.lib.d2o_prefill_attend(self.ctx, layer, view4(Q), view4(K), view4(V), n,
                                                ov, _stream_ptr()), "d2o_prefill_attend")

    def d2o_get_density(self, heads=False):
        c = self.cfg
        F = np.zeros((c.batch, c.n_layers), dtype=np.float64)
        Fh = np.zeros((c.batch, c.n_layers, c.n_q_heads), dtype=np.float64)
        self._check(self.lib.d2o_get_density(self.ctx, _np_ptr(F), _np_ptr(Fh), _stream_ptr()),
                    "d2o_get_density")
        return (F, Fh) if heads else F

    def d2o_scores_import(self, layer, scores: np.ndarray):
        scores = np.ascontiguousarray(scores, dtype=np.float32)
        assert scores.shape[:2] == (self.cfg.batch, self.cfg.n_kv_heads)
        self._check(self.lib.d2o_scores_import(self.ctx, layer, _np_ptr(scores), scores.shape[2],
                                               _stream_ptr()), "d2o_scores_import")

    def d2o_scores_export(self, layer, n):
        out = np.zeros((self.cfg.batch, self.cfg.n_kv_heads, n), dtype=np.float32)
        self._check(self.lib.d2o_scores_export(self.ctx, layer, _np_ptr(out), n, _stream_ptr()),
                    "d2o_scores_export")
        return out

    def _budget_arrays(self, budget, recent):
        b = np.ascontiguousarray(np.broadcast_to(np.asarray(budget, dtype=np.int32),
                                                 (self.cfg.batch,)))
        r = np.ascontiguousarray(np.broadcast_to(np.asarray(recent, dtype=np.int32),
                                                 (self.cfg.batch,)))
        return b, r

    def d2o_compress_layer(self, layer, K, V, budget, recent):
        b, r = self._budget_arrays(budget, recent)
        self._check(self.lib.d2o_compress_layer(self.ctx, layer, view4(K), view4(V), K.shape[2],
                                                _np_ptr(b), _np_ptr(r), _stream_ptr()),
                    "d2o_compress_layer")

    def d2o_compress_layer_heads(self, layer, K, V, budget, recent):
        """budget, recent: [B][Hkv] integer arrays (a cache size and a recent window per KV head)."""
        shape = (self.cfg.batch, self.cfg.n_kv_heads)
        b = np.ascontiguousarray(np.broadcast_to(np.asarray(budget, dtype=np.int32), shape))
        r = np.ascontiguousarray(np.broadcast_to(np.asarray(recent, dtype=np.int32), shape))
        self._check(self.lib.d2o_compress_layer_heads(self.ctx, layer, view4(K), view4(V), K.shape[2],
                                                      _np_ptr(b), _np_ptr(r), _stream_ptr()),
                    "d2o_compress_layer_heads")

    def d2o_prefill_compress(self, layer, Q, K, V, budget, recent, O=None):
        b, r = self._budget_arrays(budget, recent)
        ov = view4(O) if O is not None else _NULL_VIEW
        self._check(self.lib.d2o_prefill_compress(self.ctx, layer, view4(Q), view4(K), view4(V),
                                                  Q.shape[2], ov, _np_ptr(b), _np_ptr(r),
                                                  _stream_ptr()), "d2o_prefill_compress")

    def d2o_decode_step(self, layer, n_layers_in_call, q, k_new, v_new, out):
        self._check(self.lib.d2o_decode_step(self.ctx, layer, n_layers_in_call, view_decode(q),
                                             view_decode(k_new), view_decode(v_new),
                                             view_decode(out), _stream_ptr()), "d2o_decode_step")

    def d2o_append_chunk(self, layer, Q, K, V, O):
        """Q, O [B][Hq][m][d]; K, V [B][Hkv][m][d]: a block of m new tokens on one layer."""
        self._check(self.lib.d2o_append_chunk(self.ctx, layer, view4(Q), view4(K), view4(V), Q.shape[2],
                                              view4(O), _stream_ptr()), "d2o_append_chunk")

    def d2o_append_events(self, layer, b, kv_head, capacity):
        """(evicted positions, target positions, best similarities, passed flags) of the last block."""
        evi = np.zeros(capacity, dtype=np.int32)
        tgt = np.zeros(capacity, dtype=np.int32)
        us = np.zeros(capacity, dtype=np.float64)
        ps = np.zeros(capacity, dtype=np.uint8)
        ne = C.c_int32()
        self._check(self.lib.d2o_append_events(self.ctx, layer, b, kv_head, _np_ptr(evi), C.byref(ne),
                                               _np_ptr(tgt), _np_ptr(us), _np_ptr(ps), _stream_ptr()),
                    "d2o_append_events")
        e = ne.value
        return evi[:e], tgt[:e], us[:e], ps[:e].astype(bool)

    def d2o_decode_step_static(self, layer, n_layers_in_call, q, k_new, v_new, out):
        self._check(self.lib.d2o_decode_step_static(self.ctx, layer, n_layers_in_call, view_decode(q),
                                                    view_decode(k_new), view_decode(v_new),
                                                    view_decode(out), _stream_ptr()), "d2o_decode_step_static")

    def d2o_timing_enable(self, on):
        """False / 0: off.  True / 1: every launch.  n > 1: decode kernels every n-th launch."""
        self._check(self.lib.d2o_timing_enable(self.ctx, int(on)), "d2o_timing_enable")

    def d2o_timing_read(self, kernel: str):
        """(total milliseconds, launches) of one kernel since its last read."""
        ms, cnt = C.c_double(), C.c_int64()
        self._check(self.lib.d2o_timing_read(self.ctx, KERNEL_IDS[kernel], C.byref(ms),
                                             C.byref(cnt), _stream_ptr()), "d2o_timing_read")
        return ms.value, cnt.value

    def d2o_layer_reserve(self, layer, n, budget, recent):
        b, r = self._budget_arrays(budget, recent)
        self._check(self.lib.d2o_layer_reserve(self.ctx, layer, n, _np_ptr(b), _np_ptr(r)),
                    "d2o_layer_reserve")

    def d2o_cache_export(self, layer, b, kv_head, capacity):
        """Returns (K [count, d] fp64, V, score, pos, tau); rows in ascending position."""
        d = self.cfg.head_dim
        K = np.zeros((capacity, d), dtype=self.np_elem)
        V = np.zeros((capacity, d), dtype=self.np_elem)
        score = np.zeros(capacity, dtype=np.float64)
        pos = np.zeros(capacity, dtype=np.int32)
        count, tau = C.c_int32(), C.c_double()
        self._check(self.lib.d2o_cache_export(self.ctx, layer, b, kv_head, _np_ptr(K), _np_ptr(V),
                                              _np_ptr(score), _np_ptr(pos), C.byref(count),
                                              C.byref(tau), _stream_ptr()), "d2o_cache_export")
        n = count.value
        assert n <= capacity
        return (elems_to_f64(K[:n], self.dtype), elems_to_f64(V[:n], self.dtype), score[:n],
                pos[:n], tau.value)

    def d2o_cache_import(self, layer, b, kv_head, K, V, score, pos, tau, next_pos):
        Kb = f64_to_elems(K, self.dtype)
        Vb = f64_to_elems(V, self.dtype)
        score = np.ascontiguousarray(score, dtype=np.float64)
        pos = np.ascontiguousarray(pos, dtype=np.int32)
        self._check(self.lib.d2o_cache_import(self.ctx, layer, b, kv_head, _np_ptr(Kb), _np_ptr(Vb),
                                              _np_ptr(score), _np_ptr(pos), len(pos), float(tau),
                                              next_pos, _stream_ptr()), "d2o_cache_import")

    def d2o_candidate_misses(self):
        """Evictions of generation steps that took a token outside the predicted candidates."""
        m = C.c_int64()
        self._check(self.lib.d2o_candidate_misses(self.ctx, C.byref(m), _stream_ptr()), "d2o_candidate_misses")
        return m.value

    def d2o_last_events(self, layer):
        c = self.cfg
        ev = np.zeros((c.batch, c.n_kv_heads), dtype=np.int32)
        tg = np.zeros((c.batch, c.n_kv_heads), dtype=np.int32)
        us = np.zeros((c.batch, c.n_kv_heads), dtype=np.float64)
        self._check(self.lib.d2o_last_events(self.ctx, layer, _np_ptr(ev), _np_ptr(tg), _np_ptr(us),
                                             _stream_ptr()), "d2o_last_events")
        return ev, tg, us

    def d2o_prefill_events(self, layer, b, kv_head, n):
        ret = np.zeros(n, dtype=np.int32)
        evi = np.zeros(n, dtype=np.int32)
        tgt = np.zeros(n, dtype=np.int32)
        us = np.zeros(n, dtype=np.float64)
        ps = np.zeros(n, dtype=np.uint8)
        nr, ne = C.c_int32(), C.c_int32()
        self._check(self.lib.d2o_prefill_events(self.ctx, layer, b, kv_head, _np_ptr(ret),
                                                C.byref(nr), _np_ptr(evi), C.byref(ne), _np_ptr(tgt),
                                                _np_ptr(us), _np_ptr(ps), _stream_ptr()),
                    "d2o_prefill_events")
        r, e = nr.value, ne.value
        return ret[:r], evi[:e], tgt[:e], us[:e], ps[:e].astype(bool)


KERNEL_IDS = {"attn_fwd": 0, "colsum": 1, "select": 2, "match_filter": 3, "match_refine": 4,
              "merge": 5, "decode_attend": 6, "decode_prepare": 7, "decode_close": 8}


# ---- element conversions for host-side export / import (bit moves, no arithmetic) ----------

def elems_to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def f64_to_elems(a, dtype: str) -> np.ndarray:
    """Values must already be representable in the storage dtype."""
    a = np.ascontiguousarray(a, dtype=np.float64)
    if dtype == "bf16":
        f = a.astype(np.float32)
        bits = f.view(np.uint32)
        assert np.all((bits & 0xFFFF) == 0), "value not representable in bf16"
        return np.ascontiguousarray((bits >> 16).astype(np.uint16))
    f = a.astype(np.float32)
    assert np.all(f.astype(np.float64) == a), "value not representable in fp32"
    return np.ascontiguousarray(f)


def tensor_to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact conversion of a (bf16 / fp32) tensor to a host fp64 array."""
    return t.detach().to("cpu").to(torch.float64).numpy()
