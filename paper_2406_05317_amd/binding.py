"""Thin ctypes binding of liblococo.so (the C ABI in include/lococo.h).

Argument marshalling only: torch tensors supply device memory and the current
HIP stream; every step of the path runs inside the library's kernels.  There
is no fallback: if the shared library is missing, importing this module's
functions raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "liblococo.so")

LOCOCO_OK, LOCOCO_EINVAL, LOCOCO_EUNSUPPORTED, LOCOCO_ESTATE, LOCOCO_EHIP, LOCOCO_EWORKSPACE = range(6)
LOCOCO_F32, LOCOCO_BF16 = 0, 1
LOCOCO_IMPL_AUTO, LOCOCO_IMPL_GENERIC, LOCOCO_IMPL_MFMA = 0, 1, 2
LOCOCO_FLAG_FILTERS_PREPARED = 1
(LOCOCO_OPT_RESET, LOCOCO_OPT_SPIN_LIMIT, LOCOCO_OPT_SCAN_PER_STEP, LOCOCO_OPT_CHAIN_SYNC_DEVICE,
 LOCOCO_OPT_LOGITS_TILES, LOCOCO_OPT_MAX_RESIDENT, LOCOCO_OPT_UNFUSED_KV, LOCOCO_OPT_NO_STEP_PIPELINE) = range(8)

EXPORTS = ["lococo_plan", "lococo_workspace_bytes", "lococo_attn_only", "lococo_segment_step",
           "lococo_sequence_forward", "lococo_mix_from_logits", "lococo_last_error",
           "lococo_version", "lococo_timing_begin", "lococo_timing_end", "lococo_scan_status",
           "lococo_prepare_filters", "lococo_backward_workspace_bytes", "lococo_segment_step_backward",
           "lococo_measure_peaks", "lococo_debug_option", "lococo_describe_path",
           "lococo_segment_step_noalloc", "lococo_sequence_backward_workspace_bytes",
           "lococo_sequence_backward"]


class lococo_config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("dtype", C.c_int32), ("batch", C.c_int32),
                ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("M", C.c_int32), ("conv_width", C.c_int32), ("conv_in", C.c_int32),
                ("norm", C.c_int32), ("impl", C.c_int32), ("flags", C.c_int32),
                ("w_head_stride", C.c_int64), ("b_head_stride", C.c_int64),
                ("attn_scale", C.c_float), ("norm_eps", C.c_float)]


class lococo_cache(C.Structure):
    _fields_ = [("k", C.c_void_p * 2), ("v", C.c_void_p * 2), ("cur", C.c_int32),
                ("len", C.c_int32), ("protect", C.c_void_p), ("protect_chain_stride", C.c_int64),
                ("attn_colsum", C.c_void_p)]


class lococo_tensor(C.Structure):
    _fields_ = [("p", C.c_void_p), ("stride_b", C.c_int64), ("stride_h", C.c_int64),
                ("stride_t", C.c_int64)]


class lococo_qkvo(C.Structure):
    _fields_ = [("q", lococo_tensor), ("k", lococo_tensor), ("v", lococo_tensor),
                ("o", lococo_tensor)]


class lococo_seg(C.Structure):
    _fields_ = [("start", C.c_int64), ("len", C.c_int32), ("branch", C.c_int32),
                ("len_before", C.c_int32), ("len_after", C.c_int32), ("buf_after", C.c_int32),
                ("reserved", C.c_int32)]


class lococo_kernel_time(C.Structure):
    _fields_ = [("name", C.c_char_p), ("launches", C.c_int64), ("total_ms", C.c_double)]


class lococo_path_info(C.Structure):
    _fields_ = [("path", C.c_int32), ("compute_units", C.c_int32), ("tile_slots", C.c_int32),
                ("scan_groups", C.c_int32), ("scan_resident_limit", C.c_int32), ("position_split", C.c_int32),
                ("step_pipeline", C.c_int32), ("reserved", C.c_int32)]


class LococoError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"lococo status {status}: {message}")
        self.status = status


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2406_05317_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        cfgp, qp, cap = C.POINTER(lococo_config), C.POINTER(lococo_qkvo), C.POINTER(lococo_cache)
        L.lococo_plan.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                  C.POINTER(lococo_seg), C.POINTER(C.c_int64)]
        L.lococo_workspace_bytes.argtypes = [cfgp, C.c_int64, C.c_int32, C.c_int32,
                                             C.POINTER(C.c_size_t)]
        L.lococo_attn_only.argtypes = [cfgp, qp, C.c_int32, cap, C.c_void_p]
        L.lococo_segment_step.argtypes = [cfgp, qp, C.c_int32, C.c_void_p, C.c_void_p, cap,
                                          C.c_void_p, C.c_size_t, C.c_void_p]
        L.lococo_segment_step_noalloc.argtypes = [cfgp, qp, C.c_int32, C.c_void_p, C.c_void_p, cap, C.c_void_p]
        L.lococo_sequence_forward.argtypes = [cfgp, qp, C.c_int64, C.c_int32, C.c_void_p,
                                              C.c_void_p, cap, C.c_void_p, C.c_size_t, C.c_void_p]
        L.lococo_mix_from_logits.argtypes = [cfgp, qp, C.c_int32, C.c_void_p, cap, C.c_void_p]
        L.lococo_scan_status.argtypes = [cfgp, C.c_void_p, C.POINTER(C.c_int32)]
        L.lococo_prepare_filters.argtypes = [cfgp, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        fp = C.c_void_p
        L.lococo_backward_workspace_bytes.argtypes = [cfgp, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
        L.lococo_segment_step_backward.argtypes = [cfgp, qp, C.c_int32, C.c_void_p, C.c_void_p, cap] + [fp] * 10 + [
            C.c_void_p, C.c_size_t, C.c_void_p]
        L.lococo_sequence_backward_workspace_bytes.argtypes = [cfgp, C.c_int64, C.c_int32, C.POINTER(C.c_size_t)]
        L.lococo_sequence_backward.argtypes = [cfgp, qp, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, cap] + [
            fp] * 10 + [C.c_void_p, C.c_size_t, C.c_void_p]
        L.lococo_measure_peaks.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_double),
                                           C.POINTER(C.c_double)]
        L.lococo_debug_option.argtypes = [C.c_int32, C.c_int64]
        L.lococo_describe_path.argtypes = [cfgp, C.c_int32, C.POINTER(lococo_path_info)]
        L.lococo_timing_begin.argtypes = []
        L.lococo_timing_end.argtypes = [C.POINTER(lococo_kernel_time), C.POINTER(C.c_int32)]
        for n in EXPORTS[:6] + EXPORTS[8:]:
            getattr(L, n).restype = C.c_int
        L.lococo_last_error.restype = C.c_char_p
        L.lococo_version.restype = C.c_char_p
        _lib = L
    return _lib


def _check(status: int):
    if status != LOCOCO_OK:
        raise LococoError(status, lib().lococo_last_error().decode())


def _dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return LOCOCO_F32
    if dt == torch.bfloat16:
        return LOCOCO_BF16
    raise TypeError(f"unsupported storage dtype {dt}")


def make_config(*, dtype: torch.dtype, batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
                M: int, conv_width: int, conv_in: int = 0, norm: int = 0, impl: int = 0,
                w_head_stride: int = 0, b_head_stride: int = 0, attn_scale: float = 0.0,
                norm_eps: float = 0.0, flags: int = 0) -> lococo_config:
    return lococo_config(C.sizeof(lococo_config), _dtype_code(dtype), batch, n_q_heads, n_kv_heads,
                         head_dim, M, conv_width, conv_in, norm, impl, flags, w_head_stride,
                         b_head_stride, attn_scale, norm_eps)


def _tensor(t: torch.Tensor | None) -> lococo_tensor:
    """View of a [b, h, tokens, d] torch tensor (d contiguous)."""
    if t is None:
        return lococo_tensor(None, 0, 0, 0)
    assert t.dim() == 4 and t.stride(3) == 1, "expected [b, h, t, d] with d contiguous"
    return lococo_tensor(t.data_ptr(), t.stride(0), t.stride(1), t.stride(2))


def _qkvo(q, k, v, o) -> lococo_qkvo:
    return lococo_qkvo(_tensor(q), _tensor(k), _tensor(v), _tensor(o))


def _ptr(t: torch.Tensor | None):
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class Cache:
    """Device buffers of the double-buffered KV cache plus the host-side state."""

    def __init__(self, cfg: lococo_config, device="cuda", dtype: torch.dtype | None = None):
        dt = dtype or (torch.float32 if cfg.dtype == LOCOCO_F32 else torch.bfloat16)
        shape = (cfg.batch, cfg.n_kv_heads, cfg.M, cfg.head_dim)
        self.kbuf = [torch.zeros(shape, dtype=dt, device=device) for _ in range(2)]
        self.vbuf = [torch.zeros(shape, dtype=dt, device=device) for _ in range(2)]
        self.c = lococo_cache((C.c_void_p * 2)(self.kbuf[0].data_ptr(), self.kbuf[1].data_ptr()),
                              (C.c_void_p * 2)(self.vbuf[0].data_ptr(), self.vbuf[1].data_ptr()),
                              0, 0, None, 0, None)
        self.M, self.device = cfg.M, device
        self._protect = None
        self.attn_colsum = None
        self._chains = (cfg.batch, cfg.n_kv_heads, cfg.M)

    @property
    def len(self) -> int:
        return self.c.len

    @property
    def cur(self) -> int:
        return self.c.cur

    @property
    def k(self) -> torch.Tensor:
        return self.kbuf[self.c.cur]

    @property
    def v(self) -> torch.Tensor:
        return self.vbuf[self.c.cur]

    def set_protect(self, mask):
        """mask: None, or a bool array/tensor [M] (one mask for every chain) or [batch, n_kv_heads, M]:
        True = the slot is protected (see lococo_cache.protect in lococo.h)."""
        if mask is None:
            self._protect, self.c.protect, self.c.protect_chain_stride = None, None, 0
            return
        m = torch.as_tensor(mask).to(torch.bool).cpu()
        words = (self.M + 31) // 32
        flat = m.reshape(-1, self.M)
        bits = torch.zeros(flat.shape[0], words * 32, dtype=torch.int64)
        bits[:, :self.M] = flat.to(torch.int64)
        w = (bits.reshape(flat.shape[0], words, 32) << torch.arange(32, dtype=torch.int64)).sum(-1)
        w = torch.where(w >= 2 ** 31, w - 2 ** 32, w).to(torch.int32)
        self._protect = w.to(self.device).contiguous()
        self.c.protect = self._protect.data_ptr()
        self.c.protect_chain_stride = 0 if m.dim() == 1 else words

    def track_attention(self, on: bool = True):
        """Allocate (zeroed) or drop the fp32 [batch, n_kv_heads, M] accumulator of attention scores
        per cache slot (see lococo_cache.attn_colsum in lococo.h); read it as `self.attn_colsum`."""
        self.attn_colsum = torch.zeros(self._chains, dtype=torch.float32, device=self.device) if on else None
        self.c.attn_colsum = _ptr(self.attn_colsum)

    def load(self, k: torch.Tensor, v: torch.Tensor, length: int):
        self.kbuf[self.c.cur].copy_(k)
        self.vbuf[self.c.cur].copy_(v)
        self.c.len = length


def lococo_version() -> str:
    return lib().lococo_version().decode()


def lococo_plan(L: int, B: int, M: int, len0: int = 0, cur0: int = 0):
    """List of (start, len, branch, len_before, len_after, buf_after) tuples."""
    n = C.c_int64(0)
    _check(lib().lococo_plan(L, B, M, len0, cur0, None, C.byref(n)))
    rows = (lococo_seg * max(n.value, 1))()
    cap = C.c_int64(n.value)
    _check(lib().lococo_plan(L, B, M, len0, cur0, rows, C.byref(cap)))
    return [(r.start, r.len, r.branch, r.len_before, r.len_after, r.buf_after)
            for r in rows[:n.value]]


def lococo_workspace_bytes(cfg: lococo_config, L: int, B: int, history: bool = False) -> int:
    out = C.c_size_t(0)
    _check(lib().lococo_workspace_bytes(C.byref(cfg), L, B, int(history), C.byref(out)))
    return out.value


def lococo_attn_only(cfg, q, k, v, o, cache: Cache):
    B = q.shape[2]
    x = _qkvo(q, k, v, o)
    _check(lib().lococo_attn_only(C.byref(cfg), C.byref(x), B, C.byref(cache.c), _stream()))


def lococo_segment_step(cfg, q, k, v, o, conv_w, conv_b, cache: Cache, workspace=None):
    B = q.shape[2]
    x = _qkvo(q, k, v, o)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lococo_segment_step(C.byref(cfg), C.byref(x), B, _ptr(conv_w), _ptr(conv_b),
                                     C.byref(cache.c), _ptr(workspace), ws_bytes, _stream()))


def lococo_segment_step_noalloc(cfg, q, k, v, o, conv_w, conv_b, cache: Cache):
    """lococo_segment_step on the library's own scratch array (allocates nothing)."""
    B = q.shape[2]
    x = _qkvo(q, k, v, o)
    _check(lib().lococo_segment_step_noalloc(C.byref(cfg), C.byref(x), B, _ptr(conv_w), _ptr(conv_b),
                                             C.byref(cache.c), _stream()))


def lococo_sequence_forward(cfg, q, k, v, o, conv_w, conv_b, cache: Cache, B: int, workspace=None):
    L = q.shape[2]
    x = _qkvo(q, k, v, o)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lococo_sequence_forward(C.byref(cfg), C.byref(x), L, B, _ptr(conv_w),
                                         _ptr(conv_b), C.byref(cache.c), _ptr(workspace), ws_bytes,
                                         _stream()))


def lococo_mix_from_logits(cfg, k, v, logits, cache: Cache):
    B = k.shape[2]
    assert logits.dtype == torch.float32 and logits.is_contiguous()
    x = _qkvo(None, k, v, None)
    _check(lib().lococo_mix_from_logits(C.byref(cfg), C.byref(x), B, logits.data_ptr(),
                                        C.byref(cache.c), _stream()))


def lococo_prepare_filters(cfg, conv_w, workspace):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lococo_prepare_filters(C.byref(cfg), _ptr(conv_w), _ptr(workspace), ws_bytes, _stream()))


def lococo_backward_workspace_bytes(cfg, B: int, length: int) -> int:
    out = C.c_size_t(0)
    _check(lib().lococo_backward_workspace_bytes(C.byref(cfg), B, length, C.byref(out)))
    return out.value


def lococo_segment_step_backward(cfg, q, k, v, conv_w, conv_b, cache: Cache, d_o, d_new_k, d_new_v, d_q, d_k,
                                 d_v, d_cache_k, d_cache_v, d_conv_w, d_conv_b, workspace):
    """Gradients of one block step; `cache` is the state BEFORE the step.  All gradient tensors are
    fp32, contiguous, on the device; d_conv_w / d_conv_b are added to."""
    for t in (d_o, d_new_k, d_new_v, d_q, d_k, d_v, d_cache_k, d_cache_v, d_conv_w, d_conv_b):
        assert t is None or (t.dtype == torch.float32 and t.is_contiguous() and t.is_cuda)
    B = q.shape[2]
    x = _qkvo(q, k, v, None)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lococo_segment_step_backward(
        C.byref(cfg), C.byref(x), B, _ptr(conv_w), _ptr(conv_b), C.byref(cache.c), _ptr(d_o), _ptr(d_new_k),
        _ptr(d_new_v), _ptr(d_q), _ptr(d_k), _ptr(d_v), _ptr(d_cache_k), _ptr(d_cache_v), _ptr(d_conv_w),
        _ptr(d_conv_b), _ptr(workspace), ws_bytes, _stream()))


def lococo_sequence_backward_workspace_bytes(cfg, L: int, B: int) -> int:
    out = C.c_size_t(0)
    _check(lib().lococo_sequence_backward_workspace_bytes(C.byref(cfg), L, B, C.byref(out)))
    return out.value


def lococo_sequence_backward(cfg, q, k, v, B: int, conv_w, conv_b, cache: Cache, d_o, d_final_k, d_final_v, d_q,
                             d_k, d_v, d_cache0_k, d_cache0_v, d_conv_w, d_conv_b, workspace):
    """Gradients of a whole scan started from `cache` (left as it is).  All gradient tensors are fp32,
    contiguous, on the device; d_final_k / d_final_v may be None (zero); d_conv_w / d_conv_b are added to."""
    for t in (d_o, d_final_k, d_final_v, d_q, d_k, d_v, d_cache0_k, d_cache0_v, d_conv_w, d_conv_b):
        assert t is None or (t.dtype == torch.float32 and t.is_contiguous() and t.is_cuda)
    L = q.shape[2]
    x = _qkvo(q, k, v, None)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lococo_sequence_backward(
        C.byref(cfg), C.byref(x), L, B, _ptr(conv_w), _ptr(conv_b), C.byref(cache.c), _ptr(d_o), _ptr(d_final_k),
        _ptr(d_final_v), _ptr(d_q), _ptr(d_k), _ptr(d_v), _ptr(d_cache0_k), _ptr(d_cache0_v), _ptr(d_conv_w),
        _ptr(d_conv_b), _ptr(workspace), ws_bytes, _stream()))


def lococo_scan_status(cfg, workspace) -> int:
    """Synchronises; 0 = fine, 1 = a chain wait inside a one-launch scan gave up."""
    out = C.c_int32(0)
    _check(lib().lococo_scan_status(C.byref(cfg), _ptr(workspace), C.byref(out)))
    return out.value


def lococo_measure_peaks(scratch: torch.Tensor) -> tuple:
    """(bf16 MFMA TFLOP/s of a bare loop, GB/s of a plain copy inside `scratch`) on the current GPU."""
    tf, gbs = C.c_double(0.0), C.c_double(0.0)
    _check(lib().lococo_measure_peaks(_ptr(scratch), scratch.numel() * scratch.element_size(), _stream(),
                                      C.byref(tf), C.byref(gbs)))
    return tf.value, gbs.value


def lococo_debug_option(option: int, value: int = 0):
    """Process-wide test / measurement hook (see LOCOCO_OPT_* in lococo.h)."""
    _check(lib().lococo_debug_option(option, value))


def lococo_describe_path(cfg, B: int) -> dict:
    """Which kernels the configuration runs on, on the current device."""
    out = lococo_path_info()
    _check(lib().lococo_describe_path(C.byref(cfg), B, C.byref(out)))
    return {"path": out.path, "compute_units": out.compute_units, "tile_slots": out.tile_slots,
            "scan_groups": out.scan_groups, "scan_resident_limit": out.scan_resident_limit,
            "position_split": out.position_split, "step_pipeline": out.step_pipeline}


def lococo_timing_begin():
    _check(lib().lococo_timing_begin())


def lococo_timing_end() -> dict:
    """{kernel name: (launches, total_ms)} for the kernels launched since lococo_timing_begin."""
    rows = (lococo_kernel_time * 32)()
    n = C.c_int32(32)
    _check(lib().lococo_timing_end(rows, C.byref(n)))
    return {rows[i].name.decode(): (rows[i].launches, rows[i].total_ms) for i in range(n.value)}


def workspace(cfg, L: int, B: int, history: bool = False, device="cuda") -> torch.Tensor | None:
    """Allocate (through torch) the workspace a call with these sizes needs."""
    n = lococo_workspace_bytes(cfg, L, B, history)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device) if n else None


def config_for(w, impl: int = 0, **over) -> lococo_config:
    """lococo_config of an inputs.Workload."""
    Cc = w.C
    kw = dict(dtype=w.torch_dtype, batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads,
              head_dim=w.head_dim, M=w.M, conv_width=w.conv_width, conv_in=w.conv_in, norm=w.norm,
              impl=impl,
              w_head_stride=w.M * Cc * w.conv_width if w.per_head_filters else 0,
              b_head_stride=w.M if w.per_head_filters else 0)
    kw.update(over)
    return make_config(**kw)
