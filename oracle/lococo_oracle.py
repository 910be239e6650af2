"""ctypes front end of the CPU oracle (oracle/lococo_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg; never by the product package.  Argument
marshalling only -- every number comes out of the C++ file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lococo_oracle.cpp")
# LOCOCO_ORACLE_LIB: another build of the same source to load instead (the sanitizer job of the tests)
_LIB = os.environ.get("LOCOCO_ORACLE_LIB") or os.path.join(_HERE, "liblococo_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (generic x86-64 code: built here, run elsewhere)."""
    if os.environ.get("LOCOCO_ORACLE_LIB"):
        return _LIB                          # somebody else's build: load it as it is
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC])
    return _LIB


def build_sanitized(out_path: str) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (host code only), any
    finding fatal; loaded through LOCOCO_ORACLE_LIB with libasan preloaded."""
    subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-pthread",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
                           "-o", out_path, _SRC])
    return out_path


class Cfg(C.Structure):
    _fields_ = [("group", C.c_int32), ("head_dim", C.c_int32), ("M", C.c_int32),
                ("conv_width", C.c_int32), ("conv_in", C.c_int32), ("norm", C.c_int32),
                ("state_round", C.c_int32), ("reserved", C.c_int32),
                ("attn_scale", C.c_double), ("norm_eps", C.c_double)]


_DP = C.POINTER(C.c_double)


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        L = C.CDLL(_LIB)
        L.lococo_oracle_plan.restype = C.c_int64
        L.lococo_oracle_plan.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                         C.POINTER(C.c_int64), C.c_int64]
        L.lococo_oracle_round.restype = C.c_double
        L.lococo_oracle_round.argtypes = [C.c_double, C.c_int32]
        L.lococo_oracle_attention_block.restype = C.c_int32
        L.lococo_oracle_attention_block.argtypes = [_DP] * 5 + [C.c_int32] * 3 + [C.c_double, _DP]
        L.lococo_oracle_conv_logits.restype = C.c_int32
        L.lococo_oracle_conv_logits.argtypes = [_DP, C.c_int32, C.c_int32, _DP, _DP, C.c_int32,
                                                C.c_int32, C.c_int32, _DP]
        L.lococo_oracle_normalise.restype = C.c_int32
        L.lococo_oracle_normalise.argtypes = [_DP, C.c_int32, C.c_int32, C.c_int32, C.c_double, _DP]
        L.lococo_oracle_mix.restype = C.c_int32
        L.lococo_oracle_mix.argtypes = [_DP, _DP, C.c_int32, C.c_int32, C.c_int32, _DP]
        L.lococo_oracle_sequence_forward.restype = C.c_int32
        L.lococo_oracle_sequence_forward.argtypes = [
            C.POINTER(Cfg), C.c_int32, C.c_int32, C.c_int64, C.c_int32, _DP, _DP, _DP, _DP, _DP,
            _DP, C.POINTER(C.c_int32), _DP, C.c_int64, _DP, C.c_int64, _DP, C.c_int32]
        L.lococo_oracle_sequence_forward_protected.restype = C.c_int32
        L.lococo_oracle_sequence_forward_protected.argtypes = [
            C.POINTER(Cfg), C.c_int32, C.c_int32, C.c_int64, C.c_int32, _DP, _DP, _DP, _DP, _DP,
            _DP, C.POINTER(C.c_int32), _DP, C.c_int64, _DP, C.c_int64, _DP,
            C.POINTER(C.c_uint8), C.c_int64, _DP, C.c_int32]
        L.lococo_oracle_step_backward.restype = C.c_int32
        L.lococo_oracle_step_backward.argtypes = (
            [C.POINTER(Cfg), C.c_int32, C.c_int32, C.c_int32] + [_DP] * 5 + [C.c_int32, _DP, C.c_int64, _DP,
             C.c_int64, C.POINTER(C.c_uint8), C.c_int64] + [_DP] * 10)
        _lib = L
    return _lib


def _f64(x) -> np.ndarray:
    """Contiguous float64 numpy view/copy of a numpy array or torch tensor (exact widening)."""
    if hasattr(x, "detach"):
        import torch
        x = x.detach().to("cpu", torch.float64).numpy()
    return np.ascontiguousarray(x, dtype=np.float64)


def _p(a):
    return None if a is None else a.ctypes.data_as(_DP)


def _ok(rc):
    if rc != 0:
        raise ValueError("oracle: bad arguments")


def plan(L: int, B: int, M: int, len0: int = 0, cur0: int = 0) -> np.ndarray:
    """[n_segments, 6] int64: start, len, branch, len_before, len_after, buf_after."""
    n = lib().lococo_oracle_plan(L, B, M, len0, cur0, None, 0)
    out = np.zeros((max(n, 1), 6), dtype=np.int64)
    lib().lococo_oracle_plan(L, B, M, len0, cur0, out.ctypes.data_as(C.POINTER(C.c_int64)), n)
    return out[:n]


def round_value(x: float, mode: int) -> float:
    return lib().lococo_oracle_round(float(x), mode)


def attention_block(q, kb, vb, ck, cv, scale=None) -> np.ndarray:
    """q, kb, vb [Bn, d]; ck, cv [m, d] -> o [Bn, d] (one query head)."""
    q, kb, vb = _f64(q), _f64(kb), _f64(vb)
    Bn, d = q.shape
    ck = _f64(ck).reshape(-1, d)
    cv = _f64(cv).reshape(-1, d)
    m = ck.shape[0]
    assert kb.shape == vb.shape == (Bn, d) and cv.shape == (m, d)
    o = np.empty((Bn, d))
    _ok(lib().lococo_oracle_attention_block(_p(q), _p(kb), _p(vb), _p(ck), _p(cv), m, Bn, d,
                                            float(scale if scale is not None else d ** -0.5), _p(o)))
    return o


def conv_logits(X, Wc, bias=None, relu_input: bool = False) -> np.ndarray:
    """X [T, C], Wc [M, C, k], bias [M] or None -> W [M, T].  relu_input: the entries of X pass
    through max(., 0) first (the rectifier in front of the convolution, norm = 2)."""
    X, Wc = _f64(X), _f64(Wc)
    T, Cc = X.shape
    M, C2, k = Wc.shape
    assert C2 == Cc and k % 2 == 1
    b = None if bias is None else _f64(bias)
    W = np.empty((M, T))
    _ok(lib().lococo_oracle_conv_logits(_p(X), T, Cc, _p(Wc), _p(b), M, k, int(relu_input), _p(W)))
    return W


def normalise(W, norm: int = 0, eps: float = 1e-6) -> np.ndarray:
    W = _f64(W)
    M, T = W.shape
    w = np.empty((M, T))
    _ok(lib().lococo_oracle_normalise(_p(W), M, T, norm, eps, _p(w)))
    return w


def mix(w, Y) -> np.ndarray:
    """w [M, T], Y [T, d] -> [M, d]."""
    w, Y = _f64(w), _f64(Y)
    M, T = w.shape
    assert Y.shape[0] == T
    out = np.empty((M, Y.shape[1]))
    _ok(lib().lococo_oracle_mix(_p(w), _p(Y), M, T, Y.shape[1], _p(out)))
    return out


_ROUND = {None: 0, "none": 0, "f64": 0, "f32": 1, "bf16": 2}


def sequence_forward(q, k, v, conv_w, conv_b=None, *, B: int, M: int, conv_in: int = 0,
                     norm: int = 0, state_round="none", attn_scale: float = 0.0,
                     norm_eps: float = 1e-6, cache_k=None, cache_v=None, cache_len: int = 0,
                     logits_override=None, protect=None, attn_colsum=None, nthreads: int = 1):
    """Alg. 2 over q [b,Hq,L,d], k, v [b,Hkv,L,d].

    conv_w is [M,C,k] (shared) or [Hkv,M,C,k]; conv_b [M], [Hkv,M] or None.
    protect: None, or a boolean / 0-1 array [M] (one mask for all chains) or [b,Hkv,M]: a
    protected slot, once live, is kept as it is by every compression step and carries no weight
    in the mixing of the other slots (combination with an eviction policy, ablation on combining
    with StreamingLLM / H2O).
    attn_colsum: None, or a float64 C-contiguous array [b,Hkv,M] that is ADDED to: for every block,
    the attention probabilities its queries (all heads of the group) put on each live cache slot
    (the accumulated scores a heavy-hitter policy ranks slots by).
    Returns (o [b,Hq,L,d], cache_k [b,Hkv,M,d], cache_v, cache_len); rows of the
    caches at and beyond cache_len are zero / untouched input.
    """
    q, k, v = _f64(q), _f64(k), _f64(v)
    b, Hq, L, d = q.shape
    Hkv = k.shape[1]
    assert k.shape == v.shape == (b, Hkv, L, d) and Hq % Hkv == 0
    ck = np.zeros((b, Hkv, M, d)) if cache_k is None else _f64(cache_k).copy()
    cv = np.zeros((b, Hkv, M, d)) if cache_v is None else _f64(cache_v).copy()
    assert ck.shape == cv.shape == (b, Hkv, M, d)
    cw = None if conv_w is None else _f64(conv_w)
    w_stride = 0
    kw = 1
    if cw is not None:
        kw = cw.shape[-1]
        Cc = d * (2 if conv_in else 1)
        if cw.ndim == 4:
            assert cw.shape == (Hkv, M, Cc, kw)
            w_stride = M * Cc * kw
        else:
            assert cw.shape == (M, Cc, kw)
    cb = None if conv_b is None else _f64(conv_b)
    b_stride = 0
    if cb is not None and cb.ndim == 2:
        assert cb.shape == (Hkv, M)
        b_stride = M
    lo = None
    if logits_override is not None:
        lo = _f64(logits_override)
        assert lo.shape[1:] == (b, Hkv, M, M + B), lo.shape
    assert cw is not None or lo is not None or L + cache_len <= M
    cfg = Cfg(Hq // Hkv, d, M, kw, conv_in, norm, _ROUND[state_round], 0, attn_scale, norm_eps)
    o = np.zeros((b, Hq, L, d))
    ln = C.c_int32(cache_len)
    pr, pr_stride = None, 0
    if protect is not None:
        pr = np.ascontiguousarray(np.asarray(protect) != 0, dtype=np.uint8)
        assert pr.shape in ((M,), (b, Hkv, M)), pr.shape
        pr_stride = M if pr.ndim == 3 else 0
    if attn_colsum is not None:
        assert (isinstance(attn_colsum, np.ndarray) and attn_colsum.dtype == np.float64 and
                attn_colsum.flags.c_contiguous and attn_colsum.shape == (b, Hkv, M)), "attn_colsum: float64 [b,Hkv,M]"
    rc = lib().lococo_oracle_sequence_forward_protected(
        C.byref(cfg), b, Hkv, L, B, _p(q), _p(k), _p(v), _p(o), _p(ck), _p(cv), C.byref(ln), _p(cw),
        w_stride, _p(cb), b_stride, _p(lo),
        None if pr is None else pr.ctypes.data_as(C.POINTER(C.c_uint8)), pr_stride, _p(attn_colsum), nthreads)
    if rc != 0:
        raise ValueError("oracle: bad arguments")
    return o, ck, cv, ln.value


def step_backward(q, kb, vb, cache_k, cache_v, cache_len, conv_w, conv_b, d_o, d_new_k, d_new_v, *,
                  M: int, conv_in: int = 0, norm: int = 0, attn_scale: float = 0.0,
                  norm_eps: float = 1e-6, protect=None):
    """Gradients of one pass of the Alg. 2 loop body (storage rounding ignored).

    q, d_o [b,Hq,Bn,d]; kb, vb [b,Hkv,Bn,d]; cache_k, cache_v [b,Hkv,M,d] with cache_len live
    rows BEFORE the step; d_new_k, d_new_v [b,Hkv,M,d] gradients w.r.t. the cache AFTER the step.
    Returns dict(dq, dk, dv, d_cache_k, d_cache_v, d_conv_w, d_conv_b); the filter gradients are
    sums over chains (per kv head if conv_w is [Hkv,M,C,k]).
    """
    q, kb, vb, ck, cv = _f64(q), _f64(kb), _f64(vb), _f64(cache_k), _f64(cache_v)
    d_o, gk, gv = _f64(d_o), _f64(d_new_k), _f64(d_new_v)
    b, Hq, Bn, d = q.shape
    Hkv = kb.shape[1]
    cw = None if conv_w is None else _f64(conv_w)
    cb = None if conv_b is None else _f64(conv_b)
    w_stride = b_stride = 0
    kw = 1
    if cw is not None:
        kw = cw.shape[-1]
        if cw.ndim == 4:
            w_stride = cw.shape[1] * cw.shape[2] * cw.shape[3]
    if cb is not None and cb.ndim == 2:
        b_stride = M
    cfg = Cfg(Hq // Hkv, d, M, kw, conv_in, norm, 0, 0, attn_scale, norm_eps)
    pr, pr_stride = None, 0
    if protect is not None:
        pr = np.ascontiguousarray(np.asarray(protect) != 0, dtype=np.uint8)
        pr_stride = M if pr.ndim == 3 else 0
    out = dict(dq=np.zeros_like(q), dk=np.zeros_like(kb), dv=np.zeros_like(vb), d_cache_k=np.zeros_like(ck),
               d_cache_v=np.zeros_like(cv),
               d_conv_w=None if cw is None else np.zeros_like(cw),
               d_conv_b=None if cb is None else np.zeros_like(cb))
    rc = lib().lococo_oracle_step_backward(
        C.byref(cfg), b, Hkv, Bn, _p(q), _p(kb), _p(vb), _p(ck), _p(cv), cache_len, _p(cw), w_stride, _p(cb),
        b_stride, None if pr is None else pr.ctypes.data_as(C.POINTER(C.c_uint8)), pr_stride, _p(d_o), _p(gk),
        _p(gv), _p(out["dq"]), _p(out["dk"]), _p(out["dv"]), _p(out["d_cache_k"]), _p(out["d_cache_v"]),
        _p(out["d_conv_w"]), _p(out["d_conv_b"]))
    if rc != 0:
        raise ValueError("oracle: bad arguments")
    return out
