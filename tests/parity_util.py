"""Shared helpers of the parity tests: run the HIP path through the C ABI
binding, run the oracle on the same seeded inputs, and compare per tensor."""
from __future__ import annotations

import numpy as np
import torch

from oracle import lococo_oracle as orc
from paper_2406_05317_amd import inputs

TOL = {"f32": 1e-5, "bf16": 2e-2}   # relative, per tensor (max-norm and 2-norm)


def rel_errors(got, want):
    """(max|a-r| / max|r|, ||a-r||_2 / ||r||_2) of two arrays."""
    a = np.asarray(got, dtype=np.float64)
    r = np.asarray(want, dtype=np.float64)
    diff = a - r
    den_max = max(np.abs(r).max(), 1e-300)
    den_l2 = max(np.sqrt((r * r).sum()), 1e-300)
    return np.abs(diff).max() / den_max, np.sqrt((diff * diff).sum()) / den_l2


def assert_close(got, want, tol, what=""):
    assert np.all(np.isfinite(np.asarray(got, dtype=np.float64))), f"{what}: non-finite output"
    e_max, e_l2 = rel_errors(got, want)
    assert e_max <= tol and e_l2 <= tol, f"{what}: max-rel {e_max:.3e}, l2-rel {e_l2:.3e} > {tol}"
    return e_max, e_l2


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float64).numpy()


def oracle_forward(w: inputs.Workload, q, k, v, cw, cb, *, B=None, cache=None, nthreads=8,
                   state_round=None, protect=None):
    """Oracle scan on CPU tensors in storage dtype; state rounded to the storage grid."""
    ck = cv = None
    ln = 0
    if cache is not None:
        ck, cv, ln = cache
    return orc.sequence_forward(q, k, v, cw, cb, B=B or w.B, M=w.M, conv_in=w.conv_in, norm=w.norm,
                                state_round=state_round or w.dtype, cache_k=ck, cache_v=cv,
                                cache_len=ln, protect=protect, nthreads=nthreads)


def gpu_forward(w: inputs.Workload, q, k, v, cw, cb, *, B=None, impl=0, history=False,
                cache_init=None, step_by_step=False, protect=None):
    """HIP path through the binding.  Returns (o, cache_k, cache_v, len, cur) as CPU tensors.
    history: False / True, or an int G >= 2 for a workspace that holds a window of G blocks."""
    from paper_2406_05317_amd import binding as lb
    dev = "cuda"
    B = B or w.B
    cfg = lb.config_for(w, impl=impl)
    qd, kd, vd = q.to(dev), k.to(dev), v.to(dev)
    cwd = cw.to(dev).contiguous()
    cbd = None if cb is None else cb.to(dev).contiguous()
    od = torch.full_like(qd, float("nan"))
    cache = lb.Cache(cfg, dev)
    cache.set_protect(protect)
    if cache_init is not None:
        ck, cv, ln = cache_init
        cache.load(torch.as_tensor(ck).to(dev, w.torch_dtype), torch.as_tensor(cv).to(dev, w.torch_dtype), ln)
    L = q.shape[2]
    if step_by_step:
        ws = lb.workspace(cfg, B, B, False, dev)
        for s in range(0, L, B):
            e = min(s + B, L)
            lb.lococo_segment_step(cfg, qd[:, :, s:e], kd[:, :, s:e], vd[:, :, s:e], od[:, :, s:e],
                                   cwd, cbd, cache, ws)
    else:
        ws = lb.workspace(cfg, L, B, history, dev)
        lb.lococo_sequence_forward(cfg, qd, kd, vd, od, cwd, cbd, cache, B, ws)
        status = lb.lococo_scan_status(cfg, ws) if ws is not None else 0
        assert status == 0, f"a chain wait inside the scan launch gave up (status {status})"
    torch.cuda.synchronize()
    return od.cpu(), cache.k.cpu(), cache.v.cpu(), cache.len, cache.cur


def compare_scan(w, got, want, tol=None, what=""):
    tol = tol or TOL[w.dtype]
    o_g, ck_g, cv_g, ln_g = got[:4]
    o_w, ck_w, cv_w, ln_w = want
    assert ln_g == ln_w, f"{what}: occupancy {ln_g} != {ln_w}"
    errs = {"o": assert_close(to_np(o_g), o_w, tol, what + " O")}
    if ln_w > 0:
        errs["k"] = assert_close(to_np(ck_g)[:, :, :ln_w], ck_w[:, :, :ln_w], tol, what + " cache K")
        errs["v"] = assert_close(to_np(cv_g)[:, :, :ln_w], cv_w[:, :, :ln_w], tol, what + " cache V")
    return errs


def oracle_scan_backward(w, q, k, v, cw, cb, ck0, cv0, len0, r_o, r_k, r_v, protect, state_round="none"):
    """The oracle's step backward walked over the blocks in reverse, on the oracle's own forward states."""
    states = [(np.asarray(ck0, np.float64), np.asarray(cv0, np.float64), len0)]
    starts = list(range(0, q.shape[2], w.B))
    for s0 in starts[:-1]:
        ck, cv, m = states[-1]
        sl = slice(s0, s0 + w.B)
        _, nk, nv, ln = orc.sequence_forward(q[:, :, sl], k[:, :, sl], v[:, :, sl], cw, cb, B=w.B, M=w.M,
                                             conv_in=w.conv_in, norm=w.norm, cache_k=ck, cache_v=cv, cache_len=m,
                                             protect=protect, state_round=state_round)
        states.append((nk, nv, ln))
    out = dict(dq=np.zeros(q.shape), dk=np.zeros(k.shape), dv=np.zeros(k.shape),
               d_conv_w=None if cw is None else np.zeros(cw.shape), d_conv_b=None if cb is None else np.zeros(cb.shape))
    gk, gv = np.array(r_k, np.float64), np.array(r_v, np.float64)
    for n in reversed(range(len(starts))):
        sl = slice(starts[n], starts[n] + w.B)
        ck, cv, m = states[n]
        ref = orc.step_backward(q[:, :, sl], k[:, :, sl], v[:, :, sl], ck, cv, m, cw, cb, r_o[:, :, sl], gk, gv, M=w.M,
                                conv_in=w.conv_in, norm=w.norm, protect=protect)
        out["dq"][:, :, sl], out["dk"][:, :, sl], out["dv"][:, :, sl] = ref["dq"], ref["dk"], ref["dv"]
        if cw is not None:                       # zero from a fill step
            out["d_conv_w"] += ref["d_conv_w"]
        if cb is not None:
            out["d_conv_b"] += ref["d_conv_b"]
        gk, gv = ref["d_cache_k"], ref["d_cache_v"]
    out["d_cache0_k"], out["d_cache0_v"] = gk, gv
    return out
