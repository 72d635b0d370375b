"""ctypes binding with the names of include/lt.h.  Argument marshalling only: every step of the
path runs in the library's kernels.  Device tensors are torch tensors used as plain memory; the
stream is torch's current stream unless one is given."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch

from . import build as _build

OK, ERR_INVALID_ARG, ERR_SHAPE, ERR_CAPACITY, ERR_STATE, ERR_HIP, ERR_NOMEM = range(7)
RECENT_PER_QUERY, RECENT_FIXED = 0, 1
KERNEL_DECODE_FULL, KERNEL_DECODE_LAZY, KERNEL_APPEND = range(3)
MASK_CAUSAL, MASK_STREAMING = 0, 1
OUT_BF16, OUT_F32 = 0, 1
DECODE_AUTO, DECODE_VECTOR, DECODE_MATRIX = 0, 1, 2

EXPORTS = [
    "lt_kv_bytes", "lt_workspace_bytes", "lt_create", "lt_destroy", "lt_reset", "lt_layer_len", "lt_layer_view",
    "lt_lazy_ratio_workspace_bytes", "lt_lazy_ratio", "lt_select_lazy", "lt_append_kv", "lt_decode_attn", "lt_decode_step",
    "lt_set_split", "lt_set_shared_tail", "lt_set_decode_path", "lt_decode_plan_read", "lt_profile_enable", "lt_profile_read", "lt_status_str",
    "lt_queue_create", "lt_queue_destroy", "lt_select_push", "lt_kv_bytes_online", "lt_create_online", "lt_truncate_layer",
    "lt_lazy_ratio_lse_workspace_bytes", "lt_lazy_ratio_lse", "lt_prefill_attn", "lt_preselect_lazy",
    "lt_append_kv_ragged", "lt_seq_len", "lt_set_output_dtype", "lt_probe_read",
    "lt_reset_sequence", "lt_kv_bytes_paged", "lt_create_paged", "lt_set_block_table", "lt_decode_step_active",
    "lt_lazy_ratio_static",
]


class LtError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__("%s failed: %s (status %d)" % (what, status_str(status), status))


class Config(ctypes.Structure):
    _fields_ = [
        ("n_layers", ctypes.c_int32), ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("w_sink", ctypes.c_int32),
        ("w_recent", ctypes.c_int32), ("max_tokens", ctypes.c_int64), ("softmax_scale", ctypes.c_float),
    ]


_lib = None


def library_path() -> str:
    return _build.LIB_PATH


def load() -> ctypes.CDLL:
    """Load liblt_hip.so, building it first only when no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB_PATH):
        _build.build(force=True)            # raises if hipcc is unavailable: there is no fallback path
    lib = ctypes.CDLL(_build.LIB_PATH)
    vp, sz, i32, i64 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int64
    cfgp = ctypes.POINTER(Config)
    lib.lt_kv_bytes.argtypes = [cfgp, vp]
    lib.lt_kv_bytes.restype = sz
    lib.lt_workspace_bytes.argtypes = [cfgp]
    lib.lt_workspace_bytes.restype = sz
    lib.lt_create.argtypes = [cfgp, vp, vp, sz, vp, sz, ctypes.POINTER(vp)]
    lib.lt_create.restype = ctypes.c_int
    lib.lt_destroy.argtypes = [vp]
    lib.lt_destroy.restype = None
    lib.lt_reset.argtypes = [vp]
    lib.lt_reset.restype = ctypes.c_int
    lib.lt_layer_len.argtypes = [vp, i32, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.lt_layer_len.restype = ctypes.c_int
    lib.lt_layer_view.argtypes = [vp, i32, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(i64),
                                  ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i32)]
    lib.lt_layer_view.restype = ctypes.c_int
    lib.lt_lazy_ratio_workspace_bytes.argtypes = [cfgp, i64, i32]
    lib.lt_lazy_ratio_workspace_bytes.restype = sz
    lib.lt_lazy_ratio.argtypes = [cfgp, vp, vp, i64, i64, i64, i64, i32, ctypes.c_int, vp, sz, vp, vp, vp, vp]
    lib.lt_lazy_ratio.restype = ctypes.c_int
    lib.lt_lazy_ratio_static.argtypes = [cfgp, vp, vp, i64, i64, i64, i64, i32, ctypes.c_int, vp, vp, vp, vp]
    lib.lt_lazy_ratio_static.restype = ctypes.c_int
    lib.lt_lazy_ratio_lse_workspace_bytes.argtypes = [cfgp, i64, i32]
    lib.lt_lazy_ratio_lse_workspace_bytes.restype = sz
    lib.lt_lazy_ratio_lse.argtypes = [cfgp, vp, vp, i64, i64, i64, i64, i32, ctypes.c_int, vp, i64, i64, vp, sz, vp, vp, vp, vp]
    lib.lt_lazy_ratio_lse.restype = ctypes.c_int
    lib.lt_prefill_attn.argtypes = [cfgp, vp, vp, vp, i64, i64, i64, i64, i64, ctypes.c_int, ctypes.c_int, vp, vp, vp]
    lib.lt_prefill_attn.restype = ctypes.c_int
    lib.lt_select_lazy.argtypes = [vp, i32, i32, vp, vp]
    lib.lt_preselect_lazy.argtypes = [vp, i32, i32, i32, vp, vp]
    lib.lt_preselect_lazy.restype = ctypes.c_int
    lib.lt_select_lazy.restype = ctypes.c_int
    lib.lt_append_kv.argtypes = [vp, i32, vp, vp, i64, vp]
    lib.lt_append_kv.restype = ctypes.c_int
    lib.lt_append_kv_ragged.argtypes = [vp, i32, vp, vp, i64, vp, vp]
    lib.lt_append_kv_ragged.restype = ctypes.c_int
    lib.lt_seq_len.argtypes = [vp, i32, i32, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.lt_seq_len.restype = ctypes.c_int
    lib.lt_set_output_dtype.argtypes = [vp, ctypes.c_int]
    lib.lt_set_output_dtype.restype = ctypes.c_int
    lib.lt_decode_attn.argtypes = [vp, i32, vp, vp, vp, vp]
    lib.lt_decode_attn.restype = ctypes.c_int
    lib.lt_decode_step.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp]
    lib.lt_decode_step.restype = ctypes.c_int
    lib.lt_decode_step_active.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.lt_decode_step_active.restype = ctypes.c_int
    lib.lt_set_split.argtypes = [vp, i32, i32]
    lib.lt_set_split.restype = ctypes.c_int
    lib.lt_set_shared_tail.argtypes = [vp, i32]
    lib.lt_set_shared_tail.restype = ctypes.c_int
    lib.lt_set_decode_path.argtypes = [vp, i32]
    lib.lt_set_decode_path.restype = ctypes.c_int
    lib.lt_decode_plan_read.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_int32)]
    lib.lt_decode_plan_read.restype = ctypes.c_int
    lib.lt_profile_enable.argtypes = [vp, i32]
    lib.lt_profile_enable.restype = ctypes.c_int
    lib.lt_profile_read.argtypes = [vp, i32, ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_double)]
    lib.lt_profile_read.restype = ctypes.c_int
    lib.lt_queue_create.argtypes = [i32, ctypes.POINTER(vp)]
    lib.lt_queue_create.restype = ctypes.c_int
    lib.lt_queue_destroy.argtypes = [vp]
    lib.lt_queue_destroy.restype = None
    lib.lt_select_push.argtypes = [vp, ctypes.c_float, i32, ctypes.POINTER(i32)]
    lib.lt_select_push.restype = ctypes.c_int
    lib.lt_kv_bytes_online.argtypes = [cfgp, i32]
    lib.lt_kv_bytes_online.restype = sz
    lib.lt_create_online.argtypes = [cfgp, i32, vp, sz, vp, sz, ctypes.POINTER(vp)]
    lib.lt_create_online.restype = ctypes.c_int
    lib.lt_truncate_layer.argtypes = [vp, i32, vp]
    lib.lt_truncate_layer.restype = ctypes.c_int
    lib.lt_probe_read.argtypes = [vp, sz, vp, vp]
    lib.lt_probe_read.restype = ctypes.c_int
    lib.lt_reset_sequence.argtypes = [vp, i32]
    lib.lt_reset_sequence.restype = ctypes.c_int
    lib.lt_kv_bytes_paged.argtypes = [cfgp, vp, i32, i32]
    lib.lt_kv_bytes_paged.restype = sz
    lib.lt_create_paged.argtypes = [cfgp, vp, i32, i32, vp, sz, vp, sz, ctypes.POINTER(vp)]
    lib.lt_create_paged.restype = ctypes.c_int
    lib.lt_set_block_table.argtypes = [vp, vp, vp]
    lib.lt_set_block_table.restype = ctypes.c_int
    lib.lt_status_str.argtypes = [ctypes.c_int]
    lib.lt_status_str.restype = ctypes.c_char_p
    _lib = lib
    return lib


def status_str(status: int) -> str:
    return load().lt_status_str(int(status)).decode()


def _check(status: int, what: str) -> None:
    if status != OK:
        raise LtError(status, what)


def make_config(n_layers, batch, n_q_heads, n_kv_heads, head_dim, w_sink, w_recent, max_tokens, softmax_scale=0.0) -> Config:
    return Config(int(n_layers), int(batch), int(n_q_heads), int(n_kv_heads), int(head_dim), int(w_sink),
                  int(w_recent), int(max_tokens), float(softmax_scale))


def _mask_array(is_lazy: Sequence[int]) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(is_lazy, dtype=np.uint8))


def _dev_ptr(t: Optional[torch.Tensor], dtype, what: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError("%s must be a contiguous device tensor of %s" % (what, dtype))
    return t.data_ptr()


def _stream_ptr(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def probe_read(buf: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    """One streaming read of `buf` (any dtype, contiguous, device); `sink`: >= 256 bytes on the device."""
    if not buf.is_cuda or not buf.is_contiguous() or not sink.is_cuda or sink.numel() * sink.element_size() < 256:
        raise TypeError("buf and sink must be contiguous device tensors, sink of at least 256 bytes")
    _check(load().lt_probe_read(buf.data_ptr(), buf.numel() * buf.element_size(), sink.data_ptr(), _stream_ptr(stream)), "lt_probe_read")


def kv_bytes(cfg: Config, is_lazy) -> int:
    m = _mask_array(is_lazy)
    return int(load().lt_kv_bytes(ctypes.byref(cfg), m.ctypes.data))


def workspace_bytes(cfg: Config) -> int:
    return int(load().lt_workspace_bytes(ctypes.byref(cfg)))


def lazy_ratio_workspace_bytes(cfg: Config, n: int, w_last: int) -> int:
    return int(load().lt_lazy_ratio_workspace_bytes(ctypes.byref(cfg), int(n), int(w_last)))


def select_lazy(ratios, n_lazy: int):
    """Host-only.  Returns (is_lazy uint8 [L], order int32 [L])."""
    r = np.ascontiguousarray(np.asarray(ratios, dtype=np.float32))
    L = int(r.shape[0])
    is_lazy = np.zeros(L, dtype=np.uint8)
    order = np.zeros(L, dtype=np.int32)
    st = load().lt_select_lazy(r.ctypes.data, L, int(n_lazy), is_lazy.ctypes.data, order.ctypes.data)
    _check(st, "lt_select_lazy")
    return is_lazy, order


def preselect_lazy(is_lazy_samples, n_lazy: int):
    """Host-only.  is_lazy_samples uint8 [S, L].  Returns (is_lazy uint8 [L], count int32 [L])."""
    m = np.ascontiguousarray(np.asarray(is_lazy_samples, dtype=np.uint8))
    if m.ndim != 2:
        raise TypeError("is_lazy_samples must be [samples, layers]")
    S, L = m.shape
    is_lazy = np.zeros(L, dtype=np.uint8)
    count = np.zeros(L, dtype=np.int32)
    _check(load().lt_preselect_lazy(m.ctypes.data, S, L, int(n_lazy), is_lazy.ctypes.data, count.ctypes.data), "lt_preselect_lazy")
    return is_lazy, count


def _check_score_inputs(cfg: Config, q_last: torch.Tensor, k: torch.Tensor, n: int, w_last: int, what: str) -> None:
    """The library sees only addresses and strides: the extents of the tensors are checked here, so that a wrong n or
    a mis-shaped tensor is an error status and never a read past the end of a buffer."""
    if q_last.dtype != torch.bfloat16 or k.dtype != torch.bfloat16:
        raise TypeError("q_last and k must be bf16 tensors")
    if not q_last.is_contiguous() or k.dim() != 4 or k.stride(3) != 1:
        raise TypeError("q_last must be contiguous and k must have contiguous head_dim")
    n, w_last = int(n), int(w_last)
    if tuple(q_last.shape) != (cfg.batch, cfg.n_q_heads, w_last, cfg.head_dim):
        raise LtError(ERR_SHAPE, "%s: q_last is %s, expected [B=%d, Hq=%d, w_last=%d, %d]" % (
            what, tuple(q_last.shape), cfg.batch, cfg.n_q_heads, w_last, cfg.head_dim))
    if tuple(k.shape[:2]) != (cfg.batch, cfg.n_kv_heads) or k.shape[3] != cfg.head_dim or n < 1 or n > k.shape[2]:
        raise LtError(ERR_SHAPE, "%s: k is %s, expected [B=%d, Hkv=%d, >= n=%d, %d]" % (
            what, tuple(k.shape), cfg.batch, cfg.n_kv_heads, n, cfg.head_dim))
    if not q_last.is_cuda or q_last.device != k.device:
        raise TypeError("q_last and k must be on one GPU")


def _check_workspace(workspace: torch.Tensor, need: int, device, what: str) -> None:
    if not workspace.is_cuda or workspace.device != device or not workspace.is_contiguous():
        raise TypeError("%s: the workspace must be a contiguous tensor on the inputs' device" % what)
    if workspace.numel() * workspace.element_size() < need:
        raise LtError(ERR_CAPACITY, "%s: workspace of %d bytes, %d needed" % (what, workspace.numel() * workspace.element_size(), need))


def lazy_ratio(cfg: Config, q_last: torch.Tensor, k: torch.Tensor, n: int, w_last: int, mode: int = RECENT_PER_QUERY,
               workspace: Optional[torch.Tensor] = None, want_rho: bool = False, stream=None):
    """q_last bf16 [B,Hq,w,128]; k bf16 [B,Hkv,>=n,128] (any strides with contiguous dims).

    Returns device tensors (ratio_mean [1], ratio_seq [B], rho [B,Hq,w] or None)."""
    lib = load()
    _check_score_inputs(cfg, q_last, k, n, w_last, "lt_lazy_ratio")
    need = lazy_ratio_workspace_bytes(cfg, n, w_last)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q_last.device)
    _check_workspace(workspace, need, q_last.device, "lt_lazy_ratio")
    dev = q_last.device
    mean = torch.empty(1, dtype=torch.float32, device=dev)
    seq = torch.empty(cfg.batch, dtype=torch.float32, device=dev)
    rho = torch.empty((cfg.batch, cfg.n_q_heads, w_last), dtype=torch.float32, device=dev) if want_rho else None
    st = lib.lt_lazy_ratio(ctypes.byref(cfg), q_last.data_ptr(), k.data_ptr(), k.stride(0), k.stride(1), k.stride(2),
                           int(n), int(w_last), int(mode), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                           rho.data_ptr() if rho is not None else None, seq.data_ptr(), mean.data_ptr(), _stream_ptr(stream))
    _check(st, "lt_lazy_ratio")
    return mean, seq, rho


def lazy_ratio_static(cfg: Config, q_last: torch.Tensor, k: torch.Tensor, n: int, w_last: int, mean_out: torch.Tensor,
                      seq_out: Optional[torch.Tensor] = None, rho_out: Optional[torch.Tensor] = None,
                      mode: int = RECENT_PER_QUERY, stream=None) -> None:
    """lt_lazy_ratio_static: the same ratios with the partial results in the library's built-in scratch array.
    Nothing is allocated here either: the caller brings the outputs (fp32 device tensors: mean_out [1],
    seq_out [B] or None, rho_out [B,Hq,w] or None)."""
    _check_score_inputs(cfg, q_last, k, n, w_last, "lt_lazy_ratio_static")
    for t, shape, name in ((mean_out, (1,), "mean_out"), (seq_out, (cfg.batch,), "seq_out"),
                           (rho_out, (cfg.batch, cfg.n_q_heads, int(w_last)), "rho_out")):
        if t is None:
            continue
        if t.dtype != torch.float32 or t.device != q_last.device or not t.is_contiguous() or tuple(t.shape) != shape:
            raise LtError(ERR_SHAPE, "lt_lazy_ratio_static: %s must be a contiguous fp32 tensor %s on the inputs' device" % (name, shape))
    st = load().lt_lazy_ratio_static(ctypes.byref(cfg), q_last.data_ptr(), k.data_ptr(), k.stride(0), k.stride(1), k.stride(2),
                                     int(n), int(w_last), int(mode), rho_out.data_ptr() if rho_out is not None else None,
                                     seq_out.data_ptr() if seq_out is not None else None, mean_out.data_ptr(), _stream_ptr(stream))
    _check(st, "lt_lazy_ratio_static")


def lazy_ratio_lse_workspace_bytes(cfg: Config, n: int, w_last: int) -> int:
    return int(load().lt_lazy_ratio_lse_workspace_bytes(ctypes.byref(cfg), int(n), int(w_last)))


def lazy_ratio_lse(cfg: Config, q_last: torch.Tensor, k: torch.Tensor, n: int, w_last: int, lse_rows: torch.Tensor,
                   mode: int = RECENT_PER_QUERY, workspace: Optional[torch.Tensor] = None, want_rho: bool = False, stream=None):
    """Lazy ratio from the prefill's log-sum-exp.  lse_rows: fp32 view [B,Hq,w_last] (last dim contiguous) of the rows
    n-w_last..n-1, e.g. ``lse[:, :, n - w_last:]`` of prefill_attn's output.  Returns what lazy_ratio returns."""
    lib = load()
    _check_score_inputs(cfg, q_last, k, n, w_last, "lt_lazy_ratio_lse")
    if lse_rows.dtype != torch.float32 or not lse_rows.is_cuda or lse_rows.dim() != 3 or lse_rows.stride(2) != 1 \
            or tuple(lse_rows.shape) != (cfg.batch, cfg.n_q_heads, w_last):
        raise TypeError("lse_rows must be an fp32 device view [B, Hq, w_last] with a contiguous last dim")
    if lse_rows.device != q_last.device:
        raise TypeError("lse_rows must be on the inputs' device")
    need = lazy_ratio_lse_workspace_bytes(cfg, n, w_last)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q_last.device)
    _check_workspace(workspace, need, q_last.device, "lt_lazy_ratio_lse")
    dev = q_last.device
    mean = torch.empty(1, dtype=torch.float32, device=dev)
    seq = torch.empty(cfg.batch, dtype=torch.float32, device=dev)
    rho = torch.empty((cfg.batch, cfg.n_q_heads, w_last), dtype=torch.float32, device=dev) if want_rho else None
    st = lib.lt_lazy_ratio_lse(ctypes.byref(cfg), q_last.data_ptr(), k.data_ptr(), k.stride(0), k.stride(1), k.stride(2),
                               int(n), int(w_last), int(mode), lse_rows.data_ptr(), lse_rows.stride(0), lse_rows.stride(1),
                               workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                               rho.data_ptr() if rho is not None else None, seq.data_ptr(), mean.data_ptr(), _stream_ptr(stream))
    _check(st, "lt_lazy_ratio_lse")
    return mean, seq, rho


def prefill_attn(cfg: Config, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, n: int, mask: int = MASK_CAUSAL,
                 out_dtype=torch.bfloat16, want_lse: bool = True, stream=None):
    """q bf16 [B,Hq,n_q,128] contiguous, the queries of the last n_q of n positions (n_q = n: a whole prompt);
    k, v bf16 [B,Hkv,>=n,128] with equal strides and contiguous dims.
    Returns (out [B,Hq,n_q,128] in out_dtype, lse fp32 [B,Hq,n_q] or None)."""
    lib = load()
    for t in (q, k, v):
        if t.dtype != torch.bfloat16:
            raise TypeError("q, k, v must be bf16 tensors")
    if not q.is_contiguous() or q.dim() != 4 or k.dim() != 4 or k.stride(3) != 1 or k.stride() != v.stride():
        raise TypeError("q must be contiguous [B,Hq,n_q,128]; k and v need equal strides and contiguous head_dim")
    if out_dtype not in (torch.bfloat16, torch.float32):
        raise TypeError("out_dtype must be bfloat16 or float32")
    n_q, n = int(q.shape[2]), int(n)
    if tuple(q.shape) != (cfg.batch, cfg.n_q_heads, n_q, cfg.head_dim) or n_q < 1:
        raise LtError(ERR_SHAPE, "lt_prefill_attn: q is %s, expected [B=%d, Hq=%d, n_q, %d]" % (
            tuple(q.shape), cfg.batch, cfg.n_q_heads, cfg.head_dim))
    if tuple(k.shape[:2]) != (cfg.batch, cfg.n_kv_heads) or k.shape[3] != cfg.head_dim or tuple(v.shape) != tuple(k.shape) \
            or n < n_q or n > k.shape[2]:
        raise LtError(ERR_SHAPE, "lt_prefill_attn: k / v are %s / %s, expected [B=%d, Hkv=%d, >= n=%d, %d] with n >= n_q=%d" % (
            tuple(k.shape), tuple(v.shape), cfg.batch, cfg.n_kv_heads, n, cfg.head_dim, n_q))
    if not q.is_cuda or q.device != k.device or q.device != v.device:
        raise TypeError("q, k and v must be on one GPU")
    out = torch.empty((cfg.batch, cfg.n_q_heads, n_q, cfg.head_dim), dtype=out_dtype, device=q.device)
    lse = torch.empty((cfg.batch, cfg.n_q_heads, n_q), dtype=torch.float32, device=q.device) if want_lse else None
    st = lib.lt_prefill_attn(ctypes.byref(cfg), q.data_ptr(), k.data_ptr(), v.data_ptr(), k.stride(0), k.stride(1), k.stride(2),
                             int(n), n_q, int(mask), OUT_F32 if out_dtype == torch.float32 else OUT_BF16, out.data_ptr(),
                             lse.data_ptr() if lse is not None else None, _stream_ptr(stream))
    _check(st, "lt_prefill_attn")
    return out, lse


class SelectQueue:
    """The max-priority queue of the online procedure (host only)."""

    def __init__(self, capacity: int):
        handle = ctypes.c_void_p()
        _check(load().lt_queue_create(int(capacity), ctypes.byref(handle)), "lt_queue_create")
        self._h = handle

    def push(self, ratio: float, layer: int) -> int:
        """Returns the layer that left the queue, or -1."""
        popped = ctypes.c_int32(-1)
        _check(load().lt_select_push(self._h, float(ratio), int(layer), ctypes.byref(popped)), "lt_select_push")
        return popped.value

    def close(self):
        if getattr(self, "_h", None):
            load().lt_queue_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def kv_bytes_online(cfg: Config, n_full: int) -> int:
    return int(load().lt_kv_bytes_online(ctypes.byref(cfg), int(n_full)))


def kv_bytes_paged(cfg: Config, is_lazy, page_tokens: int, n_pages: int) -> int:
    mask = _mask_array(is_lazy)
    return int(load().lt_kv_bytes_paged(ctypes.byref(cfg), mask.ctypes.data, int(page_tokens), int(n_pages)))


class Context:
    """Owns the torch tensors used as KV slab and workspace, and the library's host-side context.

    With a lazy mask: lt_create.  With `n_full_online` instead: lt_create_online (layers take storage on
    demand and turn lazy through truncate_layer).  With a lazy mask and `paged=(page_tokens, n_pages)`:
    lt_create_paged (full layers are pools of pages behind set_block_table)."""

    def __init__(self, cfg: Config, is_lazy=None, device="cuda:0", n_full_online: Optional[int] = None, guard_bytes: int = 0,
                 paged=None):
        lib = load()
        self.cfg = cfg
        online = n_full_online is not None
        self.paged = tuple(int(x) for x in paged) if paged is not None else None
        if online and self.paged:
            raise ValueError("a context is either online or paged")
        if online:
            kvb = kv_bytes_online(cfg, n_full_online)
        else:
            self.is_lazy = _mask_array(is_lazy)
            if self.is_lazy.shape[0] != cfg.n_layers:
                raise ValueError("is_lazy needs one entry per layer")
            kvb = kv_bytes_paged(cfg, self.is_lazy, *self.paged) if self.paged else kv_bytes(cfg, self.is_lazy)
        wsb = workspace_bytes(cfg)
        if kvb == 0 or wsb == 0:
            raise LtError(ERR_INVALID_ARG, "lt_kv_bytes / lt_workspace_bytes")
        self.device = torch.device(device)
        # testing aid: `guard_bytes` (a multiple of 256) of a known pattern on both sides of the slab and the
        # workspace; check_guards() tells whether anything wrote there
        self._guard = int(guard_bytes)
        if self._guard % 256:
            raise ValueError("guard_bytes must be a multiple of 256")
        make = (lambda nbytes: torch.full((nbytes,), 0xA5, dtype=torch.uint8, device=self.device)) if self._guard else \
            (lambda nbytes: torch.empty(nbytes, dtype=torch.uint8, device=self.device))
        self._slab_all = make(kvb + 2 * self._guard)
        self._ws_all = make(wsb + 2 * self._guard)
        self.kv_slab = self._slab_all[self._guard: self._guard + kvb]
        self.workspace = self._ws_all[self._guard: self._guard + wsb]
        handle = ctypes.c_void_p()
        if online:
            st = lib.lt_create_online(ctypes.byref(cfg), int(n_full_online), self.kv_slab.data_ptr(), kvb,
                                      self.workspace.data_ptr(), wsb, ctypes.byref(handle))
            _check(st, "lt_create_online")
        elif self.paged:
            st = lib.lt_create_paged(ctypes.byref(cfg), self.is_lazy.ctypes.data, self.paged[0], self.paged[1],
                                     self.kv_slab.data_ptr(), kvb, self.workspace.data_ptr(), wsb, ctypes.byref(handle))
            _check(st, "lt_create_paged")
        else:
            st = lib.lt_create(ctypes.byref(cfg), self.is_lazy.ctypes.data, self.kv_slab.data_ptr(), kvb,
                               self.workspace.data_ptr(), wsb, ctypes.byref(handle))
            _check(st, "lt_create")
        self._h = handle
        self.out_dtype = torch.float32
        # LT_DECODE_PATH=vector|matrix forces one of the two decode kernels for every context of the process (the test
        # suite runs its decode tests once more on each); unset or "auto": the library chooses per launch
        forced = os.environ.get("LT_DECODE_PATH", "auto")
        if forced != "auto":
            self.set_decode_path({"vector": DECODE_VECTOR, "matrix": DECODE_MATRIX}[forced])

    def check_guards(self) -> bool:
        """True when the guard bands around the slab and the workspace still hold their pattern."""
        g = self._guard
        if g == 0:
            return True
        bands = (self._slab_all[:g], self._slab_all[-g:], self._ws_all[:g], self._ws_all[-g:])
        return all(bool((b == 0xA5).all().item()) for b in bands)

    def set_block_table(self, table, stream=None):
        """table: int32 [B, max_pages] (host; numpy or CPU tensor), -1 = no page."""
        if not self.paged:
            raise LtError(ERR_STATE, "lt_set_block_table (context is not paged)")
        max_pages = -(-int(self.cfg.max_tokens) // self.paged[0])
        t = np.ascontiguousarray(np.asarray(table, dtype=np.int32))
        if t.shape != (self.cfg.batch, max_pages):
            raise LtError(ERR_SHAPE, "lt_set_block_table (table must be [B, ceil(max_tokens / page_tokens)])")
        _check(load().lt_set_block_table(self._h, t.ctypes.data, _stream_ptr(stream)), "lt_set_block_table")

    def reset_sequence(self, sequence: int):
        _check(load().lt_reset_sequence(self._h, int(sequence)), "lt_reset_sequence")

    def truncate_layer(self, layer: int, stream=None):
        _check(load().lt_truncate_layer(self._h, int(layer), _stream_ptr(stream)), "lt_truncate_layer")

    def close(self):
        """Destroys the host-side context and lets go of the slab and the workspace (views handed out by
        layer_tensors keep the memory alive for as long as they live)."""
        if getattr(self, "_h", None):
            load().lt_destroy(self._h)
            self._h = None
            self._slab_all = self._ws_all = self.kv_slab = self.workspace = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reset(self):
        _check(load().lt_reset(self._h), "lt_reset")

    def layer_len(self, layer: int):
        total, stored = ctypes.c_int64(), ctypes.c_int64()
        _check(load().lt_layer_len(self._h, int(layer), ctypes.byref(total), ctypes.byref(stored)), "lt_layer_len")
        return total.value, stored.value

    def layer_view(self, layer: int):
        k, v = ctypes.c_void_p(), ctypes.c_void_p()
        sb, sh, cap, lazy = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int32()
        _check(load().lt_layer_view(self._h, int(layer), ctypes.byref(k), ctypes.byref(v), ctypes.byref(sb),
                                    ctypes.byref(sh), ctypes.byref(cap), ctypes.byref(lazy)), "lt_layer_view")
        return {"k": k.value, "v": v.value, "stride_b": sb.value, "stride_h": sh.value, "capacity": cap.value,
                "is_lazy": bool(lazy.value)}

    def layer_tensors(self, layer: int):
        """Views of a layer's K and V blocks inside the slab: bf16 [B, Hkv, capacity, 128]; for a full layer
        of a paged context its pools, bf16 [n_pages, Hkv, page_tokens, 128]."""
        view = self.layer_view(layer)
        shape = (self.cfg.batch, self.cfg.n_kv_heads, view["capacity"], self.cfg.head_dim)
        if self.paged and not view["is_lazy"]:
            shape = (self.paged[1], self.cfg.n_kv_heads, self.paged[0], self.cfg.head_dim)
        count = int(np.prod(shape))
        base = self.kv_slab.data_ptr()
        out = []
        for key in ("k", "v"):
            off = view[key] - base
            out.append(self.kv_slab[off: off + 2 * count].view(torch.bfloat16).view(shape))
        return out[0], out[1]

    def append_kv(self, layer: int, k_new: torch.Tensor, v_new: torch.Tensor, stream=None):
        kp, vp = _dev_ptr(k_new, torch.bfloat16, "k_new"), _dev_ptr(v_new, torch.bfloat16, "v_new")
        expect = (self.cfg.batch, self.cfg.n_kv_heads, k_new.shape[2] if k_new.dim() == 4 else -1, self.cfg.head_dim)
        if tuple(k_new.shape) != expect or tuple(v_new.shape) != expect:
            raise LtError(ERR_SHAPE, "lt_append_kv (k_new / v_new must be [B,Hkv,n_new,128])")
        st = load().lt_append_kv(self._h, int(layer), kp, vp, int(k_new.shape[2]), _stream_ptr(stream))
        _check(st, "lt_append_kv")

    def append_kv_ragged(self, layer: int, k_new: torch.Tensor, v_new: torch.Tensor, lengths, stream=None):
        """k_new / v_new: bf16 [B,Hkv,n_max,128] (padded); lengths: B token counts, each in 0..n_max."""
        kp, vp = _dev_ptr(k_new, torch.bfloat16, "k_new"), _dev_ptr(v_new, torch.bfloat16, "v_new")
        expect = (self.cfg.batch, self.cfg.n_kv_heads, k_new.shape[2] if k_new.dim() == 4 else -1, self.cfg.head_dim)
        if tuple(k_new.shape) != expect or tuple(v_new.shape) != expect:
            raise LtError(ERR_SHAPE, "lt_append_kv_ragged (k_new / v_new must be [B,Hkv,n_max,128])")
        n = np.ascontiguousarray(np.asarray(lengths, dtype=np.int64))
        if n.shape != (self.cfg.batch,):
            raise LtError(ERR_SHAPE, "lt_append_kv_ragged (one length per sequence)")
        st = load().lt_append_kv_ragged(self._h, int(layer), kp, vp, int(k_new.shape[2]), n.ctypes.data, _stream_ptr(stream))
        _check(st, "lt_append_kv_ragged")

    def seq_len(self, layer: int, sequence: int):
        """(tokens appended, entries stored) of one sequence of a layer."""
        total, stored = ctypes.c_int64(0), ctypes.c_int64(0)
        _check(load().lt_seq_len(self._h, int(layer), int(sequence), ctypes.byref(total), ctypes.byref(stored)), "lt_seq_len")
        return total.value, stored.value

    def set_output_dtype(self, dtype):
        """torch.float32 (default) or torch.bfloat16 for the `out` of decode_attn / decode_step."""
        if dtype not in (torch.float32, torch.bfloat16):
            raise TypeError("output dtype must be float32 or bfloat16")
        _check(load().lt_set_output_dtype(self._h, OUT_F32 if dtype == torch.float32 else OUT_BF16), "lt_set_output_dtype")
        self.out_dtype = dtype

    def decode_attn(self, layer: int, q: torch.Tensor, out: Optional[torch.Tensor] = None,
                    lse: Optional[torch.Tensor] = None, want_lse: bool = False, stream=None):
        qp = _dev_ptr(q, torch.bfloat16, "q")
        if tuple(q.shape) != (self.cfg.batch, self.cfg.n_q_heads, self.cfg.head_dim):
            raise LtError(ERR_SHAPE, "lt_decode_attn (q must be [B,Hq,128])")
        if out is None:
            out = torch.empty((self.cfg.batch, self.cfg.n_q_heads, self.cfg.head_dim), dtype=self.out_dtype, device=q.device)
        if lse is None and want_lse:
            lse = torch.empty((self.cfg.batch, self.cfg.n_q_heads), dtype=torch.float32, device=q.device)
        st = load().lt_decode_attn(self._h, int(layer), qp, _dev_ptr(out, self.out_dtype, "out"),
                                   _dev_ptr(lse, torch.float32, "lse"), _stream_ptr(stream))
        _check(st, "lt_decode_attn")
        return (out, lse) if (want_lse or lse is not None) else out

    def decode_step(self, layer: int, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                    out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None, want_lse: bool = False, stream=None,
                    active=None):
        """Fused append of one token + attention.  k_new / v_new: bf16 [B,Hkv,1,128] or [B,Hkv,128].
        active: optional B flags (host); sequences with a zero flag sit the step out (lt_decode_step_active)."""
        qp = _dev_ptr(q, torch.bfloat16, "q")
        kp, vp = _dev_ptr(k_new, torch.bfloat16, "k_new"), _dev_ptr(v_new, torch.bfloat16, "v_new")
        if tuple(q.shape) != (self.cfg.batch, self.cfg.n_q_heads, self.cfg.head_dim):
            raise LtError(ERR_SHAPE, "lt_decode_step (q must be [B,Hq,128])")
        if k_new.numel() != self.cfg.batch * self.cfg.n_kv_heads * self.cfg.head_dim or v_new.numel() != k_new.numel():
            raise LtError(ERR_SHAPE, "lt_decode_step (k_new / v_new must hold one token: [B,Hkv,128])")
        if out is None:
            out = torch.empty((self.cfg.batch, self.cfg.n_q_heads, self.cfg.head_dim), dtype=self.out_dtype, device=q.device)
        if lse is None and want_lse:
            lse = torch.empty((self.cfg.batch, self.cfg.n_q_heads), dtype=torch.float32, device=q.device)
        if active is not None:
            flags = np.ascontiguousarray(np.asarray(active, dtype=np.uint8))
            if flags.shape != (self.cfg.batch,):
                raise LtError(ERR_SHAPE, "lt_decode_step_active (one flag per sequence)")
            st = load().lt_decode_step_active(self._h, int(layer), qp, kp, vp, flags.ctypes.data, _dev_ptr(out, self.out_dtype, "out"),
                                              _dev_ptr(lse, torch.float32, "lse"), _stream_ptr(stream))
            _check(st, "lt_decode_step_active")
            return (out, lse) if (want_lse or lse is not None) else out
        st = load().lt_decode_step(self._h, int(layer), qp, kp, vp, _dev_ptr(out, self.out_dtype, "out"),
                                   _dev_ptr(lse, torch.float32, "lse"), _stream_ptr(stream))
        _check(st, "lt_decode_step")
        return (out, lse) if (want_lse or lse is not None) else out

    def set_split(self, keys_full: int = 0, keys_lazy: int = 0):
        _check(load().lt_set_split(self._h, int(keys_full), int(keys_lazy)), "lt_set_split")

    def set_decode_path(self, path: int = 0):
        """DECODE_AUTO, DECODE_VECTOR or DECODE_MATRIX."""
        _check(load().lt_set_decode_path(self._h, int(path)), "lt_set_decode_path")

    def decode_plan(self, layer: int) -> dict:
        """Layout of the layer's most recent decode launch: keys_per_block, n_splits, tail_begin (-1 = no shared
        tail), matrix_cores."""
        plan = (ctypes.c_int32 * 4)()
        _check(load().lt_decode_plan_read(self._h, int(layer), plan), "lt_decode_plan_read")
        return {"keys_per_block": plan[0], "n_splits": plan[1], "tail_begin": plan[2], "matrix_cores": bool(plan[3])}

    def set_shared_tail(self, on: bool = True):
        _check(load().lt_set_shared_tail(self._h, 1 if on else 0), "lt_set_shared_tail")

    def profile_enable(self, on: bool = True):
        _check(load().lt_profile_enable(self._h, 1 if on else 0), "lt_profile_enable")

    def profile_read(self, kernel: int):
        n, ms = ctypes.c_int64(), ctypes.c_double()
        _check(load().lt_profile_read(self._h, int(kernel), ctypes.byref(n), ctypes.byref(ms)), "lt_profile_read")
        return n.value, ms.value
