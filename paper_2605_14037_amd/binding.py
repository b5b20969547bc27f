"""Thin ctypes binding of include/spkv.h: argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch supplies device
memory (the arena and the tensors) and the current stream.
"""

from __future__ import annotations

import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

OK, E_INVAL, E_STATE, E_CAPACITY, E_HIP, E_NOMEM, E_DEVICE = 0, -1, -2, -3, -4, -5, -6
OPT_ITEM_TARGET, OPT_KERNEL_TIMING, OPT_SPLIT_ONLY, OPT_SINK_TOKENS, OPT_MERGE_WAVES = 1, 2, 3, 4, 5
OPT_STEP_LAUNCHES = 6
MAX_BATCH, PAGE_TOKENS = 512, 64

EXPORTED_SYMBOLS = [
    "spkv_cache_required_bytes", "spkv_cache_create", "spkv_cache_destroy", "spkv_cache_grow",
    "spkv_cache_reset",
    "spkv_append", "spkv_decode_attention", "spkv_decode_attention_static", "spkv_decode_step",
    "spkv_decode_chunk",
    "spkv_decode_step_predict_workspace_bytes", "spkv_decode_step_predict", "spkv_score_chunk",
    "spkv_prefill_workspace_bytes", "spkv_prefill_attention",
    "spkv_soft_gated_workspace_bytes", "spkv_soft_gated_attention", "spkv_cache_release_sequence", "spkv_utility_logits", "spkv_cache_safe_steps", "spkv_cache_advance", "spkv_cache_stats", "spkv_cache_kept_positions",
    "spkv_cache_threshold_logit", "spkv_cache_set_tau", "spkv_cache_prune", "spkv_cache_set_option", "spkv_cache_read_kernel_timing",
    "spkv_debug_layout_offset", "spkv_debug_copy", "spkv_debug_read", "spkv_strerror",
]


class SPKVConfig(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("window", C.c_int32), ("page_tokens", C.c_int32),
                ("tau", C.c_float), ("max_context", C.c_int32),
                ("max_total_kept_tokens", C.c_int64)]


class SPKVStats(C.Structure):
    _fields_ = [("total_tokens", C.c_int64), ("evicted_tokens", C.c_int64),
                ("window_tokens", C.c_int64), ("kept_tokens", C.c_int64),
                ("gate_on_tokens", C.c_int64), ("density_evicted", C.c_double),
                ("density_all", C.c_double), ("kept_kv_bytes", C.c_int64),
                ("dense_kv_bytes", C.c_int64), ("pool_pages_used", C.c_int64),
                ("pool_pages_total", C.c_int64), ("arena_bytes", C.c_int64),
                ("device_error", C.c_int32), ("n_work_items", C.c_int32),
                ("n_work_items_last_call", C.c_int32), ("reserved_", C.c_int32)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class SPKVError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


def library_path():
    return os.path.join(HERE, "libspkv.so")


def load_library():
    """Load libspkv.so once and declare the prototypes of include/spkv.h."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it first "
                           "(python -m paper_2605_14037_amd.build); there is no fallback path")
    lib = C.CDLL(path)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    P = C.POINTER
    lib.spkv_cache_required_bytes.restype = C.c_size_t
    lib.spkv_cache_required_bytes.argtypes = [P(SPKVConfig)]
    lib.spkv_cache_create.restype = C.c_int
    lib.spkv_cache_create.argtypes = [P(SPKVConfig), vp, C.c_size_t, vp, P(vp)]
    lib.spkv_cache_destroy.restype = C.c_int
    lib.spkv_cache_destroy.argtypes = [vp]
    lib.spkv_cache_grow.restype = C.c_int
    lib.spkv_cache_grow.argtypes = [vp, P(SPKVConfig), vp, C.c_size_t, vp]
    lib.spkv_cache_reset.restype = C.c_int
    lib.spkv_cache_reset.argtypes = [vp, vp]
    lib.spkv_append.restype = C.c_int
    lib.spkv_append.argtypes = [vp, vp, vp, vp, P(i32), vp]
    lib.spkv_decode_attention.restype = C.c_int
    lib.spkv_decode_attention.argtypes = [vp, vp, vp, vp, f32, vp]
    lib.spkv_decode_attention_static.restype = C.c_int
    lib.spkv_decode_attention_static.argtypes = [vp, vp, vp, vp, f32, vp]
    lib.spkv_decode_step.restype = C.c_int
    lib.spkv_decode_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, f32, vp]
    lib.spkv_decode_step_predict_workspace_bytes.restype = C.c_size_t
    lib.spkv_decode_step_predict_workspace_bytes.argtypes = [i32, i32]
    lib.spkv_decode_step_predict.restype = C.c_int
    lib.spkv_decode_step_predict.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp,
                                             vp, vp, C.c_size_t, f32, vp]
    lib.spkv_decode_chunk.restype = C.c_int
    lib.spkv_decode_chunk.argtypes = [vp, vp, vp, vp, vp, P(i32), vp, vp, f32, vp]
    lib.spkv_score_chunk.restype = C.c_int
    lib.spkv_score_chunk.argtypes = [vp, vp, vp, vp, P(i32), vp, vp, f32, vp]
    lib.spkv_prefill_workspace_bytes.restype = C.c_size_t
    lib.spkv_prefill_workspace_bytes.argtypes = [vp, i32, i64]
    lib.spkv_prefill_attention.restype = C.c_int
    lib.spkv_prefill_attention.argtypes = [vp, vp, vp, vp, vp, P(i32), vp, vp, f32, vp, C.c_size_t, vp]
    lib.spkv_soft_gated_workspace_bytes.restype = C.c_size_t
    lib.spkv_soft_gated_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
    lib.spkv_soft_gated_attention.restype = C.c_int
    lib.spkv_soft_gated_attention.argtypes = [vp, vp, vp, vp, P(i32), i32, i32, i32, i32, i32, vp, vp,
                                              f32, vp, C.c_size_t, vp]
    lib.spkv_cache_release_sequence.restype = C.c_int
    lib.spkv_cache_release_sequence.argtypes = [vp, i32, vp]
    lib.spkv_utility_logits.restype = C.c_int
    lib.spkv_utility_logits.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp]
    lib.spkv_cache_prune.restype = C.c_int
    lib.spkv_cache_prune.argtypes = [vp, vp]
    lib.spkv_cache_safe_steps.restype = C.c_int
    lib.spkv_cache_safe_steps.argtypes = [vp, vp, P(i64)]
    lib.spkv_cache_advance.restype = C.c_int
    lib.spkv_cache_advance.argtypes = [vp, i64]
    lib.spkv_cache_stats.restype = C.c_int
    lib.spkv_cache_stats.argtypes = [vp, P(SPKVStats), P(i32), vp]
    lib.spkv_cache_kept_positions.restype = C.c_int
    lib.spkv_cache_kept_positions.argtypes = [vp, i32, i32, P(i32), i32, P(i32), vp]
    lib.spkv_cache_threshold_logit.restype = C.c_int
    lib.spkv_cache_threshold_logit.argtypes = [vp, P(f32)]
    lib.spkv_cache_set_tau.restype = C.c_int
    lib.spkv_cache_set_tau.argtypes = [vp, f32]
    lib.spkv_cache_set_option.restype = C.c_int
    lib.spkv_cache_set_option.argtypes = [vp, i32, i64]
    lib.spkv_cache_read_kernel_timing.restype = C.c_int
    lib.spkv_cache_read_kernel_timing.argtypes = [vp, P(f32), i32, P(i32)]
    lib.spkv_debug_layout_offset.restype = i64
    lib.spkv_debug_layout_offset.argtypes = [i32, i32, i32, i32]
    lib.spkv_debug_copy.restype = C.c_int
    lib.spkv_debug_copy.argtypes = [vp, vp, C.c_size_t, vp]
    lib.spkv_debug_read.restype = C.c_int
    lib.spkv_debug_read.argtypes = [vp, C.c_size_t, i32, i64, i64, i64, i32, vp, vp]
    lib.spkv_strerror.restype = C.c_char_p
    lib.spkv_strerror.argtypes = [C.c_int]
    _LIB = lib
    return lib


def strerror(code):
    return load_library().spkv_strerror(int(code)).decode()


def required_bytes(cfg: SPKVConfig) -> int:
    return int(load_library().spkv_cache_required_bytes(C.byref(cfg)))


def layout_offset(head_dim, is_v, kidx, d) -> int:
    return int(load_library().spkv_debug_layout_offset(head_dim, int(is_v), kidx, d))


def debug_copy(dst: torch.Tensor, src: torch.Tensor):
    """Plain copy kernel of known traffic (src.nbytes read + written); see spkv_debug_copy."""
    nbytes = src.numel() * src.element_size()
    if not (dst.is_cuda and src.is_cuda and dst.is_contiguous() and src.is_contiguous()
            and dst.numel() * dst.element_size() == nbytes):
        raise ValueError("debug_copy: need contiguous cuda tensors of equal byte size")
    _check(load_library().spkv_debug_copy(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()),
                                          nbytes, _stream()), "spkv_debug_copy")


def debug_read(src: torch.Tensor, run_bytes, first_run, n_runs, stride, n_workgroups, sink):
    """Plain streaming read with the decode kernel's launch shape (spkv_debug_read)."""
    if not (src.is_cuda and src.is_contiguous() and sink.is_cuda and sink.is_contiguous()
            and sink.numel() * sink.element_size() >= n_workgroups * 1024):
        raise ValueError("debug_read: need contiguous cuda tensors, sink of n_workgroups KB")
    _check(load_library().spkv_debug_read(C.c_void_p(src.data_ptr()), src.numel() * src.element_size(),
                                          int(run_bytes), int(first_run), int(n_runs), int(stride),
                                          int(n_workgroups), C.c_void_p(sink.data_ptr()), _stream()),
           "spkv_debug_read")


def soft_gated_attention(q, k, v, util_logits, cu_seqlens, window=128, sm_scale=0.0, out=None,
                         want_lse=False, workspace=None):
    """Soft-gated attention forward over packed sequences (spkv_soft_gated_attention).
    q: bf16 [total, H_q, D]; k, v: bf16 [total, H_kv, D]; util_logits: fp32 [total, H_kv]."""
    lib = load_library()
    total, Hq, D = q.shape
    Hkv = k.shape[1]
    batch = len(cu_seqlens) - 1
    cu = (C.c_int32 * (batch + 1))(*[int(x) for x in cu_seqlens])
    if cu[batch] != total:
        raise ValueError("cu_seqlens does not cover the rows")
    qp = _dev_ptr(q, torch.bfloat16, (total, Hq, D), "q")
    kp = _dev_ptr(k, torch.bfloat16, (total, Hkv, D), "k")
    vp = _dev_ptr(v, torch.bfloat16, (total, Hkv, D), "v")
    fp = _dev_ptr(util_logits, torch.float32, (total, Hkv), "util_logits")
    n_max = max(cu[b + 1] - cu[b] for b in range(batch))
    if workspace is None:
        need = int(lib.spkv_soft_gated_workspace_bytes(batch, Hkv, D, int(window), max(n_max, 1)))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    if out is None:
        out = torch.empty_like(q)
    op = _dev_ptr(out, torch.bfloat16, (total, Hq, D), "out")
    lse = torch.empty((total, Hq), dtype=torch.float32, device=q.device) if want_lse else None
    lp = _dev_ptr(lse, torch.float32, (total, Hq), "lse") if lse is not None else None
    _check(lib.spkv_soft_gated_attention(qp, kp, vp, fp, cu, batch, Hq, Hkv, D, int(window), op, lp,
                                         float(sm_scale), workspace.data_ptr(), workspace.numel(),
                                         _stream()), "spkv_soft_gated_attention")
    return (out, lse) if want_lse else out


def utility_logits(hidden, w1, b1, w2, b2, out=None, workspace=None):
    """Pre-sigmoid utility logits of the two-layer predictor (spkv_utility_logits)."""
    n, d_model = hidden.shape
    d_hidden, n_heads = w1.shape[0], w2.shape[0]
    hp = _dev_ptr(hidden, torch.bfloat16, (n, d_model), "hidden")
    w1p = _dev_ptr(w1, torch.bfloat16, (d_hidden, d_model), "w1")
    w2p = _dev_ptr(w2, torch.bfloat16, (n_heads, d_hidden), "w2")
    b1p = _dev_ptr(b1, torch.float32, (d_hidden,), "b1") if b1 is not None else None
    b2p = _dev_ptr(b2, torch.float32, (n_heads,), "b2") if b2 is not None else None
    if out is None:
        out = torch.empty(n, n_heads, dtype=torch.float32, device=hidden.device)
    if workspace is None:
        workspace = torch.empty(max(1, n * d_hidden), dtype=torch.float32, device=hidden.device)
    op = _dev_ptr(out, torch.float32, (n, n_heads), "logits")
    _check(load_library().spkv_utility_logits(hp, w1p, b1p, w2p, b2p, op,
                                              C.c_void_p(workspace.data_ptr()), n, d_model,
                                              d_hidden, n_heads, _stream()), "spkv_utility_logits")
    return out


def _check(code, where):
    if code != OK:
        raise SPKVError(code, where)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev_ptr(t: torch.Tensor, dtype, shape, name):
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous() or tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: need a contiguous cuda {dtype} tensor of shape {tuple(shape)}, "
                         f"got {t.dtype} {tuple(t.shape)} on {t.device}")
    return C.c_void_p(t.data_ptr())


class SPKVCache:
    """One attention layer's SP-KV cache on the current CUDA (HIP) device."""

    def __init__(self, batch, n_q_heads, n_kv_heads, head_dim, max_context,
                 max_total_kept_tokens, window=128, tau=0.5, device="cuda"):
        self.lib = load_library()
        self.cfg = SPKVConfig(batch, n_q_heads, n_kv_heads, head_dim, window, 0, tau,
                              max_context, max_total_kept_tokens)
        nbytes = required_bytes(self.cfg)
        if nbytes == 0:
            raise SPKVError(E_INVAL, "spkv_cache_required_bytes")
        self.device = torch.device(device)
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.handle = C.c_void_p()
        _check(self.lib.spkv_cache_create(C.byref(self.cfg), C.c_void_p(self.arena.data_ptr()),
                                          nbytes, _stream(), C.byref(self.handle)),
               "spkv_cache_create")

    def grow(self, max_context=None, max_total_kept_tokens=None):
        """Move the cache into a new, larger arena (spkv_cache_grow).  The old arena is
        released once the copy has completed."""
        old = self.cfg
        cfg = SPKVConfig(old.batch, old.n_q_heads, old.n_kv_heads, old.head_dim, old.window, 0,
                         old.tau,
                         old.max_context if max_context is None else int(max_context),
                         old.max_total_kept_tokens if max_total_kept_tokens is None
                         else int(max_total_kept_tokens))
        nbytes = required_bytes(cfg)
        if nbytes == 0:
            raise SPKVError(E_INVAL, "spkv_cache_required_bytes")
        arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        _check(self.lib.spkv_cache_grow(self.handle, C.byref(cfg), C.c_void_p(arena.data_ptr()),
                                        nbytes, _stream()), "spkv_cache_grow")
        torch.cuda.current_stream(self.device).synchronize()    # the old arena is read until here
        self.arena, self.cfg = arena, cfg

    def close(self):
        if getattr(self, "handle", None) is not None and self.handle.value:
            torch.cuda.synchronize(self.device)
            self.lib.spkv_cache_destroy(self.handle)
            self.handle = C.c_void_p()
        self.arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- write path
    def make_cu(self, cu_seqlens):
        """cu_seqlens as the C array spkv_append takes (build once, reuse every step)."""
        return (C.c_int32 * (self.cfg.batch + 1))(*[int(x) for x in cu_seqlens])

    def append(self, k, v, util_logits, cu_seqlens):
        cfg = self.cfg
        cu = cu_seqlens if isinstance(cu_seqlens, C.Array) else self.make_cu(cu_seqlens)
        total = cu[cfg.batch]
        if total == 0:
            _check(self.lib.spkv_append(self.handle, None, None, None, cu, _stream()), "spkv_append")
            return
        kp = _dev_ptr(k, torch.bfloat16, (total, cfg.n_kv_heads, cfg.head_dim), "k")
        vp = _dev_ptr(v, torch.bfloat16, (total, cfg.n_kv_heads, cfg.head_dim), "v")
        fp = _dev_ptr(util_logits, torch.float32, (total, cfg.n_kv_heads), "util_logits")
        _check(self.lib.spkv_append(self.handle, kp, vp, fp, cu, _stream()), "spkv_append")

    # ---- read path
    def decode_attention(self, q, out=None, lse=None, sm_scale=0.0, want_lse=False):
        cfg = self.cfg
        shape = (cfg.batch, cfg.n_q_heads, cfg.head_dim)
        qp = _dev_ptr(q, torch.bfloat16, shape, "q")
        if out is None:
            out = torch.empty(shape, dtype=torch.bfloat16, device=q.device)
        op = _dev_ptr(out, torch.bfloat16, shape, "out")
        if lse is None and want_lse:
            lse = torch.empty(shape[:2], dtype=torch.float32, device=q.device)
        lp = _dev_ptr(lse, torch.float32, shape[:2], "lse") if lse is not None else None
        _check(self.lib.spkv_decode_attention(self.handle, qp, op, lp, float(sm_scale), _stream()),
               "spkv_decode_attention")
        return (out, lse) if lse is not None else out

    def decode_attention_static(self, q, out, lse=None, sm_scale=0.0):
        """spkv_decode_attention_static: partials in the library's static device array; the
        caller passes every buffer (nothing is allocated here either)."""
        cfg = self.cfg
        shape = (cfg.batch, cfg.n_q_heads, cfg.head_dim)
        qp = _dev_ptr(q, torch.bfloat16, shape, "q")
        op = _dev_ptr(out, torch.bfloat16, shape, "out")
        lp = _dev_ptr(lse, torch.float32, shape[:2], "lse") if lse is not None else None
        _check(self.lib.spkv_decode_attention_static(self.handle, qp, op, lp, float(sm_scale),
                                                     _stream()), "spkv_decode_attention_static")
        return out

    def decode_step(self, k, v, util_logits, q, out=None, lse=None, sm_scale=0.0, want_lse=False):
        """Append one token per sequence and decode, fused (spkv_decode_step)."""
        cfg = self.cfg
        kv_shape = (cfg.batch, cfg.n_kv_heads, cfg.head_dim)
        shape = (cfg.batch, cfg.n_q_heads, cfg.head_dim)
        kp = _dev_ptr(k, torch.bfloat16, kv_shape, "k")
        vp = _dev_ptr(v, torch.bfloat16, kv_shape, "v")
        fp = _dev_ptr(util_logits, torch.float32, kv_shape[:2], "util_logits")
        qp = _dev_ptr(q, torch.bfloat16, shape, "q")
        if out is None:
            out = torch.empty(shape, dtype=torch.bfloat16, device=q.device)
        op = _dev_ptr(out, torch.bfloat16, shape, "out")
        if lse is None and want_lse:
            lse = torch.empty(shape[:2], dtype=torch.float32, device=q.device)
        lp = _dev_ptr(lse, torch.float32, shape[:2], "lse") if lse is not None else None
        _check(self.lib.spkv_decode_step(self.handle, kp, vp, fp, qp, op, lp, float(sm_scale),
                                         _stream()), "spkv_decode_step")
        return (out, lse) if lse is not None else out

    def decode_step_predict(self, hidden, w1, b1, w2, b2, k, v, q, out=None, lse=None,
                            util_logits=None, workspace=None, sm_scale=0.0, want_lse=False):
        """Fused step whose gate logits come from the utility predictor, computed inside the
        step's two launches (spkv_decode_step_predict).  Returns (out, util_logits) or
        (out, lse, util_logits)."""
        cfg = self.cfg
        kv_shape = (cfg.batch, cfg.n_kv_heads, cfg.head_dim)
        shape = (cfg.batch, cfg.n_q_heads, cfg.head_dim)
        d_model, d_hidden = hidden.shape[1], w1.shape[0]
        hp = _dev_ptr(hidden, torch.bfloat16, (cfg.batch, d_model), "hidden")
        w1p = _dev_ptr(w1, torch.bfloat16, (d_hidden, d_model), "w1")
        w2p = _dev_ptr(w2, torch.bfloat16, (cfg.n_kv_heads, d_hidden), "w2")
        b1p = _dev_ptr(b1, torch.float32, (d_hidden,), "b1") if b1 is not None else None
        b2p = _dev_ptr(b2, torch.float32, (cfg.n_kv_heads,), "b2") if b2 is not None else None
        kp = _dev_ptr(k, torch.bfloat16, kv_shape, "k")
        vp = _dev_ptr(v, torch.bfloat16, kv_shape, "v")
        qp = _dev_ptr(q, torch.bfloat16, shape, "q")
        if out is None:
            out = torch.empty(shape, dtype=torch.bfloat16, device=q.device)
        op = _dev_ptr(out, torch.bfloat16, shape, "out")
        if lse is None and want_lse:
            lse = torch.empty(shape[:2], dtype=torch.float32, device=q.device)
        lp = _dev_ptr(lse, torch.float32, shape[:2], "lse") if lse is not None else None
        if util_logits is None:
            util_logits = torch.empty(kv_shape[:2], dtype=torch.float32, device=q.device)
        fp = _dev_ptr(util_logits, torch.float32, kv_shape[:2], "util_logits")
        if workspace is None:
            need = self.lib.spkv_decode_step_predict_workspace_bytes(cfg.batch, d_hidden)
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
        if workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous():
            raise ValueError("workspace must be a contiguous uint8 device tensor")
        _check(self.lib.spkv_decode_step_predict(self.handle, hp, w1p, b1p, w2p, b2p, d_model,
                                                 d_hidden, kp, vp, qp, op, lp, fp,
                                                 workspace.data_ptr(), workspace.numel(),
                                                 float(sm_scale), _stream()),
               "spkv_decode_step_predict")
        return (out, lse, util_logits) if lse is not None else (out, util_logits)

    def decode_chunk(self, k, v, util_logits, q, cu_seqlens, out=None, lse=None, sm_scale=0.0,
                     want_lse=False):
        """Append up to 16 tokens per sequence and return each one's attention output
        (spkv_decode_chunk)."""
        cfg = self.cfg
        cu = cu_seqlens if isinstance(cu_seqlens, C.Array) else self.make_cu(cu_seqlens)
        total = cu[cfg.batch]
        if total == 0:
            _check(self.lib.spkv_decode_chunk(self.handle, None, None, None, None, cu, None, None,
                                              float(sm_scale), _stream()), "spkv_decode_chunk")
            return None
        kv_shape = (total, cfg.n_kv_heads, cfg.head_dim)
        shape = (total, cfg.n_q_heads, cfg.head_dim)
        kp = _dev_ptr(k, torch.bfloat16, kv_shape, "k")
        vp = _dev_ptr(v, torch.bfloat16, kv_shape, "v")
        fp = _dev_ptr(util_logits, torch.float32, kv_shape[:2], "util_logits")
        qp = _dev_ptr(q, torch.bfloat16, shape, "q")
        if out is None:
            out = torch.empty(shape, dtype=torch.bfloat16, device=q.device)
        op = _dev_ptr(out, torch.bfloat16, shape, "out")
        if lse is None and want_lse:
            lse = torch.empty(shape[:2], dtype=torch.float32, device=q.device)
        lp = _dev_ptr(lse, torch.float32, shape[:2], "lse") if lse is not None else None
        _check(self.lib.spkv_decode_chunk(self.handle, kp, vp, fp, qp, cu, op, lp, float(sm_scale),
                                          _stream()), "spkv_decode_chunk")
        return (out, lse) if lse is not None else out

    def score_chunk(self, k, v, q, cu_seqlens, out=None, lse=None, sm_scale=0.0, want_lse=False):
        """Attention outputs of up to 16 draft tokens per sequence, the cache left unchanged
        (spkv_score_chunk)."""
        cfg = self.cfg
        cu = cu_seqlens if isinstance(cu_seqlens, C.Array) else self.make_cu(cu_seqlens)
        total = cu[cfg.batch]
        if total == 0:
            _check(self.lib.spkv_score_chunk(self.handle, None, None, None, cu, None, None,
                                             float(sm_scale), _stream()), "spkv_score_chunk")
            return None
        kv_shape = (total, cfg.n_kv_heads, cfg.head_dim)
        shape = (total, cfg.n_q_heads, cfg.head_dim)
        kp = _dev_ptr(k, torch.bfloat16, kv_shape, "k")
        vp = _dev_ptr(v, torch.bfloat16, kv_shape, "v")
        qp = _dev_ptr(q, torch.bfloat16, shape, "q")
        if out is None:
            out = torch.empty(shape, dtype=torch.bfloat16, device=q.device)
        op = _dev_ptr(out, torch.bfloat16, shape, "out")
        if lse is None and want_lse:
            lse = torch.empty(shape[:2], dtype=torch.float32, device=q.device)
        lp = _dev_ptr(lse, torch.float32, shape[:2], "lse") if lse is not None else None
        _check(self.lib.spkv_score_chunk(self.handle, kp, vp, qp, cu, op, lp, float(sm_scale),
                                         _stream()), "spkv_score_chunk")
        return (out, lse) if lse is not None else out

    def prefill_workspace_bytes(self, max_tokens_per_sequence, max_total_tokens):
        return int(self.lib.spkv_prefill_workspace_bytes(self.handle, int(max_tokens_per_sequence),
                                                         int(max_total_tokens)))

    def prefill_attention(self, k, v, util_logits, q, cu_seqlens, workspace=None, out=None,
                          lse=None, sm_scale=0.0, want_lse=False):
        """Append any number of tokens per sequence and return each one's attention output
        (spkv_prefill_attention).  workspace: uint8 device tensor of at least
        prefill_workspace_bytes(max n_b, sum n_b) bytes; allocated here if None."""
        cfg = self.cfg
        cu = cu_seqlens if isinstance(cu_seqlens, C.Array) else self.make_cu(cu_seqlens)
        total = cu[cfg.batch]
        if total == 0:
            _check(self.lib.spkv_prefill_attention(self.handle, None, None, None, None, cu, None,
                                                   None, float(sm_scale), None, 0, _stream()),
                   "spkv_prefill_attention")
            return None
        kv_shape = (total, cfg.n_kv_heads, cfg.head_dim)
        shape = (total, cfg.n_q_heads, cfg.head_dim)
        kp = _dev_ptr(k, torch.bfloat16, kv_shape, "k")
        vp = _dev_ptr(v, torch.bfloat16, kv_shape, "v")
        fp = _dev_ptr(util_logits, torch.float32, kv_shape[:2], "util_logits")
        qp = _dev_ptr(q, torch.bfloat16, shape, "q")
        if workspace is None:
            n_max = max(cu[b + 1] - cu[b] for b in range(cfg.batch))
            workspace = torch.empty(self.prefill_workspace_bytes(n_max, total), dtype=torch.uint8,
                                    device=q.device)
        if workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous():
            raise ValueError("workspace must be a contiguous uint8 device tensor")
        if out is None:
            out = torch.empty(shape, dtype=torch.bfloat16, device=q.device)
        op = _dev_ptr(out, torch.bfloat16, shape, "out")
        if lse is None and want_lse:
            lse = torch.empty(shape[:2], dtype=torch.float32, device=q.device)
        lp = _dev_ptr(lse, torch.float32, shape[:2], "lse") if lse is not None else None
        _check(self.lib.spkv_prefill_attention(self.handle, kp, vp, fp, qp, cu, op, lp,
                                               float(sm_scale), workspace.data_ptr(),
                                               workspace.numel(), _stream()),
               "spkv_prefill_attention")
        return (out, lse) if lse is not None else out

    # ---- bookkeeping
    def reset(self):
        _check(self.lib.spkv_cache_reset(self.handle, _stream()), "spkv_cache_reset")

    def release_sequence(self, b):
        _check(self.lib.spkv_cache_release_sequence(self.handle, int(b), _stream()),
               "spkv_cache_release_sequence")

    def stats(self, with_kept_len=False):
        st = SPKVStats()
        n = self.cfg.batch * self.cfg.n_kv_heads
        buf = (C.c_int32 * n)()
        _check(self.lib.spkv_cache_stats(self.handle, C.byref(st), buf, _stream()),
               "spkv_cache_stats")
        if with_kept_len:
            return st, [list(buf[b * self.cfg.n_kv_heads:(b + 1) * self.cfg.n_kv_heads])
                        for b in range(self.cfg.batch)]
        return st

    def kept_positions(self, b, h):
        cap = max(1, self.cfg.max_context)
        buf = (C.c_int32 * cap)()
        n = C.c_int32()
        _check(self.lib.spkv_cache_kept_positions(self.handle, b, h, buf, cap, C.byref(n),
                                                  _stream()), "spkv_cache_kept_positions")
        return list(buf[:n.value])

    def threshold_logit(self):
        th = C.c_float()
        _check(self.lib.spkv_cache_threshold_logit(self.handle, C.byref(th)),
               "spkv_cache_threshold_logit")
        return th.value

    def safe_steps(self):
        """Single-token steps guaranteed to fit (spkv_cache_safe_steps; synchronises)."""
        n = C.c_int64()
        _check(self.lib.spkv_cache_safe_steps(self.handle, _stream(), C.byref(n)),
               "spkv_cache_safe_steps")
        return n.value

    def advance(self, n_steps):
        """Account for n_steps steps executed by graph replays (spkv_cache_advance)."""
        _check(self.lib.spkv_cache_advance(self.handle, int(n_steps)), "spkv_cache_advance")

    def prune(self):
        """Drop every kept pair whose logit fails the current threshold (spkv_cache_prune)."""
        _check(self.lib.spkv_cache_prune(self.handle, _stream()), "spkv_cache_prune")

    def set_tau(self, tau):
        _check(self.lib.spkv_cache_set_tau(self.handle, float(tau)), "spkv_cache_set_tau")

    def set_option(self, option, value):
        _check(self.lib.spkv_cache_set_option(self.handle, option, int(value)),
               "spkv_cache_set_option")

    def read_kernel_timing(self, cap=8192):
        buf = (C.c_float * cap)()
        n = C.c_int32()
        _check(self.lib.spkv_cache_read_kernel_timing(self.handle, buf, cap, C.byref(n)),
               "spkv_cache_read_kernel_timing")
        return list(buf[:n.value])
