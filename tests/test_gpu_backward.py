"""GPU parity of the backward pass of one block step against the CPU oracle's backward (itself
pinned by finite differences of the forward oracle), single steps in every branch and variant and
a scan of several steps walked in reverse."""
import numpy as np
import pytest
import torch

from oracle import lococo_oracle as orc
from paper_2406_05317_amd import binding as lb
from paper_2406_05317_amd import inputs

pytestmark = pytest.mark.gpu


def _rel(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-30))


def _gpu_step_backward(w, cfg, q, k, v, cw, cb, ck, cv, m, d_o, gk, gv, dW, dB, protect=None):
    dev = "cuda"
    cache = lb.Cache(cfg, dev)
    cache.load(torch.as_tensor(ck).to(dev, w.torch_dtype), torch.as_tensor(cv).to(dev, w.torch_dtype), m)
    cache.set_protect(protect)
    f32 = lambda x: torch.as_tensor(np.asarray(x), dtype=torch.float32).to(dev).contiguous()
    out = dict(dq=torch.full(q.shape, float("nan"), device=dev), dk=torch.full(k.shape, float("nan"), device=dev),
               dv=torch.full(v.shape, float("nan"), device=dev),
               d_cache_k=torch.full(ck.shape, float("nan"), device=dev),
               d_cache_v=torch.full(cv.shape, float("nan"), device=dev))
    ws = torch.empty(max(lb.lococo_backward_workspace_bytes(cfg, q.shape[2], m), 256), dtype=torch.uint8, device=dev)
    lb.lococo_segment_step_backward(cfg, q.to(dev), k.to(dev), v.to(dev), None if cw is None else cw.to(dev),
                                    None if cb is None else cb.to(dev), cache, f32(d_o), f32(gk), f32(gv),
                                    out["dq"], out["dk"], out["dv"], out["d_cache_k"], out["d_cache_v"], dW, dB, ws)
    torch.cuda.synchronize()
    return {n: t.cpu().numpy() for n, t in out.items()}


CASES = [
    dict(name="f32 compress", dtype="f32", batch=2, n_q_heads=4, n_kv_heads=2, head_dim=32, B=16, M=24, m=24,
         conv_width=5),
    dict(name="f32 partial cache", dtype="f32", batch=1, n_q_heads=2, n_kv_heads=2, head_dim=16, B=12, M=20, m=14,
         conv_width=3),
    dict(name="f32 fill", dtype="f32", batch=1, n_q_heads=2, n_kv_heads=1, head_dim=16, B=6, M=20, m=5,
         conv_width=3),
    dict(name="bf16 relu-sum", dtype="bf16", batch=1, n_q_heads=2, n_kv_heads=2, head_dim=64, B=32, M=48, m=48,
         conv_width=7, norm=1, bias_sigma=0.5),
    dict(name="f32 kv channels per-head", dtype="f32", batch=2, n_q_heads=2, n_kv_heads=2, head_dim=8, B=10, M=12,
         m=12, conv_width=3, conv_in=1, per_head_filters=True, bias_sigma=0.3),
    dict(name="bf16 protected", dtype="bf16", batch=1, n_q_heads=4, n_kv_heads=2, head_dim=128, B=40, M=64, m=64,
         conv_width=15, protect=True),
    # the Eq. 5 contractions on the matrix cores (bf16, head_dim 128, keys-only filters; impl = AUTO)
    dict(name="mfma protected", dtype="bf16", batch=1, n_q_heads=4, n_kv_heads=2, head_dim=128, B=40, M=64, m=64,
         conv_width=15, protect=True, impl=0),
    dict(name="mfma ragged per-head", dtype="bf16", batch=2, n_q_heads=2, n_kv_heads=2, head_dim=128, B=100, M=160,
         m=160, conv_width=15, per_head_filters=True, bias_sigma=0.4, impl=0),     # T = 260, slots padded to 192
    dict(name="mfma partial cache relu-sum width 21", dtype="bf16", batch=1, n_q_heads=2, n_kv_heads=2, head_dim=128,
         B=70, M=128, m=90, conv_width=21, norm=1, bias_sigma=0.5, impl=0),
    dict(name="mfma several tiles grouped heads", dtype="bf16", batch=3, n_q_heads=2, n_kv_heads=1, head_dim=128,
         B=256, M=256, m=256, conv_width=15, impl=0),                              # 4 position x 2 slot tiles
    dict(name="mfma fill step", dtype="bf16", batch=2, n_q_heads=4, n_kv_heads=2, head_dim=128, B=24, M=96, m=40,
         conv_width=15, impl=0),
    dict(name="mfma head_dim 64 (plain contractions only)", dtype="bf16", batch=1, n_q_heads=2, n_kv_heads=2,
         head_dim=64, B=40, M=64, m=64, conv_width=7, bias_sigma=0.3, impl=0),
    dict(name="mfma [K|V] filters width 21 relu-sum per-head", dtype="bf16", batch=2, n_q_heads=4, n_kv_heads=2,
         head_dim=128, B=72, M=160, m=160, conv_width=21, conv_in=1, norm=1, per_head_filters=True, bias_sigma=0.4,
         impl=0),                                                                  # the compressor as the paper prints it
    dict(name="mfma [K|V] filters partial cache", dtype="bf16", batch=1, n_q_heads=2, n_kv_heads=1, head_dim=128,
         B=100, M=128, m=60, conv_width=15, conv_in=1, impl=0),
    dict(name="mfma width 3", dtype="bf16", batch=1, n_q_heads=1, n_kv_heads=1, head_dim=128, B=33, M=32, m=20,
         conv_width=3, impl=0),
]


@pytest.mark.parametrize("case", CASES, ids=[c["name"] for c in CASES])
def test_step_backward_matches_the_oracle(case):
    c = dict(case)
    c.pop("name")
    m, use_protect, impl = c.pop("m"), c.pop("protect", False), c.pop("impl", 1)
    w = inputs.Workload(name="bwd", L=c["B"], seed=11, conv_gain=3.0, **c)
    rng = np.random.default_rng(3)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    chains = (w.batch, w.n_kv_heads, w.M, w.head_dim)
    ck = torch.as_tensor(rng.standard_normal(chains) * 0.5).to(w.torch_dtype)
    cv = torch.as_tensor(rng.standard_normal(chains) * 0.5).to(w.torch_dtype)
    ck[:, :, m:], cv[:, :, m:] = 0, 0
    d_o = rng.standard_normal(q.shape)
    gk, gv = rng.standard_normal(chains), rng.standard_normal(chains)
    ln = min(w.M, m + w.B)
    gk[:, :, ln:], gv[:, :, ln:] = 0.0, 0.0
    protect = (rng.random((w.batch, w.n_kv_heads, w.M)) < 0.2) if use_protect else None
    want = orc.step_backward(q, k, v, ck, cv, m, cw, cb, d_o, gk, gv, M=w.M, conv_in=w.conv_in, norm=w.norm,
                             protect=protect)
    cfg = lb.config_for(w, impl=impl)
    dW = torch.zeros(cw.shape, dtype=torch.float32, device="cuda")
    dB = None if cb is None else torch.zeros(cb.shape, dtype=torch.float32, device="cuda")
    got = _gpu_step_backward(w, cfg, q, k, v, cw, cb, ck, cv, m, d_o, gk, gv, dW, dB, protect)
    got["d_conv_w"], got["d_conv_b"] = dW.cpu().numpy(), None if dB is None else dB.cpu().numpy()
    errs = {}
    for n in ("dq", "dk", "dv", "d_cache_k", "d_cache_v", "d_conv_w", "d_conv_b"):
        if want[n] is None:
            continue
        if m + w.B <= w.M and n in ("d_conv_w", "d_conv_b"):
            assert not got[n].any()
            continue
        if n == "d_conv_b" and w.norm == 0:
            # a softmax row does not change when its bias does: the gradient is zero up to rounding
            assert np.abs(want[n]).max() < 1e-12
            assert np.abs(got[n]).max() < 1e-5 * np.abs(want["d_conv_w"]).max()
            continue
        errs[n] = _rel(got[n], want[n])
        assert errs[n] < 2e-4, (n, errs[n])          # fp32 sums of up to ~1e3 terms against double
    assert not got["d_cache_k"][:, :, m:].any() and not got["d_cache_v"][:, :, m:].any()
    print(case["name"], {n: f"{e:.1e}" for n, e in errs.items()})


def test_scan_backward_in_reverse_matches_the_oracle_and_a_directional_difference():
    """Three block steps (fill, compress, compress): forward on the GPU keeping the cache states,
    backward step by step in reverse, filter gradients collected in one buffer.  Checked against
    the oracle's backward walked the same way, and the filter gradient against a finite
    difference of the ORACLE forward along a random direction."""
    w = inputs.Workload(name="bwdscan", dtype="f32", batch=1, n_q_heads=2, n_kv_heads=2, head_dim=16, L=36, B=12,
                        M=16, conv_width=5, seed=4, conv_gain=3.0)
    rng = np.random.default_rng(8)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    r_o = rng.standard_normal(q.shape)
    r_k, r_v = rng.standard_normal((1, 2, w.M, 16)), rng.standard_normal((1, 2, w.M, 16))

    def loss(cw_):
        o, ck, cv, _ = orc.sequence_forward(q, k, v, cw_, cb, B=w.B, M=w.M)
        return (o * r_o).sum() + (ck * r_k).sum() + (cv * r_v).sum()

    # forward states from the oracle (the GPU forward agrees to 1e-5, tested elsewhere)
    states = [(np.zeros((1, 2, w.M, 16)), np.zeros((1, 2, w.M, 16)), 0)]
    for s0 in range(0, w.L, w.B):
        ck, cv, m = states[-1]
        _, nk, nv, ln = orc.sequence_forward(q[:, :, s0:s0 + w.B], k[:, :, s0:s0 + w.B], v[:, :, s0:s0 + w.B], cw, cb,
                                             B=w.B, M=w.M, cache_k=ck, cache_v=cv, cache_len=m)
        states.append((nk, nv, ln))
    cfg = lb.config_for(w, impl=1)
    dW = torch.zeros(cw.shape, dtype=torch.float32, device="cuda")
    want_dW = np.zeros(cw.shape)
    gk, gv = r_k.copy(), r_v.copy()
    wk, wv = r_k.copy(), r_v.copy()
    for n in reversed(range(w.L // w.B)):
        sl = slice(n * w.B, (n + 1) * w.B)
        ck, cv, m = states[n]
        got = _gpu_step_backward(w, cfg, q[:, :, sl].contiguous(), k[:, :, sl].contiguous(), v[:, :, sl].contiguous(),
                                 cw, None, torch.as_tensor(ck), torch.as_tensor(cv), m, r_o[:, :, sl], gk, gv, dW, None)
        ref = orc.step_backward(q[:, :, sl], k[:, :, sl], v[:, :, sl], ck, cv, m, cw, None, r_o[:, :, sl], wk, wv, M=w.M)
        if ref["d_conv_w"] is not None:
            want_dW += ref["d_conv_w"]
        gk, gv = got["d_cache_k"], got["d_cache_v"]
        wk, wv = ref["d_cache_k"], ref["d_cache_v"]
        assert _rel(got["dq"], ref["dq"]) < 2e-4 and _rel(got["dk"], ref["dk"]) < 2e-4
    assert _rel(dW.cpu().numpy(), want_dW) < 2e-4
    direction = rng.standard_normal(cw.shape)
    eps = 1e-5
    cw64 = cw.double().numpy()
    fd = (loss(cw64 + eps * direction) - loss(cw64 - eps * direction)) / (2 * eps)
    assert abs((dW.cpu().numpy() * direction).sum() - fd) < 2e-4 * max(1.0, abs(fd))
