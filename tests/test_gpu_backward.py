"""GPU parity of the backward pass of one block step against the CPU oracle's backward (itself
pinned by finite differences of the forward oracle), single steps in every branch and variant and
a scan of several steps walked in reverse."""
import numpy as np
import pytest
import torch

from oracle import lococo_oracle as orc
from paper_2406_05317_amd import binding as lb
from paper_2406_05317_amd import inputs
from parity_util import oracle_scan_backward

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


def _draw_step(i):
    rng = np.random.default_rng(17000 + i)
    ch = lambda xs: xs[int(rng.integers(len(xs)))]
    dtype = ch(["bf16", "bf16", "f32"])
    d = ch([64, 128, 128, 128]) if dtype == "bf16" else ch([8, 16, 32, 64])
    M = ch([12, 20, 32, 48, 64, 96, 128, 160, 192, 256])
    Hkv = ch([1, 2, 3])
    case = dict(dtype=dtype, head_dim=d, M=M, B=ch([1, 6, 24, 33, 40, 64, 100, 128, 200]),
                conv_width=ch([1, 3, 5, 7, 15, 21]), norm=ch([0, 0, 1]), conv_in=ch([0, 0, 1]),
                per_head_filters=ch([False, False, True]), bias_sigma=ch([0.0, 0.4]), n_kv_heads=Hkv,
                n_q_heads=Hkv * ch([1, 2, 4]), batch=ch([1, 2]), conv_gain=ch([1.0, 3.0]))
    return case, ch([M, M, int(rng.integers(0, M + 1))]), ch([0, 1]), ch([False, False, True]), rng


@pytest.mark.parametrize("i", range(40))
def test_step_backward_on_a_drawn_case(i):
    """A seeded sweep over storage type, sizes, occupancy, filter width, normalisation, convolution input, filter
    sharing, grouped heads, protected slots and kernel family: every gradient against the oracle's."""
    case, m, impl, use_protect, rng = _draw_step(i)
    w = inputs.Workload(name=f"bwd{i}", L=case["B"], seed=17000 + i, **case)
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
    what = f"{w} m={m} impl={impl} protect={use_protect}"
    for n in ("dq", "dk", "dv", "d_cache_k", "d_cache_v", "d_conv_w", "d_conv_b"):
        if want[n] is None:
            continue
        if m + w.B <= w.M and n in ("d_conv_w", "d_conv_b"):
            assert not got[n].any(), (n, what)
        elif n == "d_conv_b" and w.norm == 0:
            assert np.abs(got[n]).max() < 1e-5 * max(np.abs(want["d_conv_w"]).max(), 1e-30), (n, what)
        else:
            assert np.all(np.isfinite(got[n])), (n, what)
            assert _rel(got[n], want[n]) < 2e-4, (n, _rel(got[n], want[n]), what)
    assert not got["d_cache_k"][:, :, m:].any() and not got["d_cache_v"][:, :, m:].any()


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


# ---- the whole scan in one call ---------------------------------------------------------------

def _gpu_scan_backward(w, cfg, q, k, v, cw, cb, ck0, cv0, len0, r_o, r_k, r_v, protect):
    dev = "cuda"
    cache = lb.Cache(cfg, dev)
    cache.load(torch.as_tensor(ck0).to(dev, w.torch_dtype), torch.as_tensor(cv0).to(dev, w.torch_dtype), len0)
    cache.set_protect(protect)
    before = (cache.k.clone(), cache.v.clone(), cache.len, cache.cur)
    f32 = lambda x: None if x is None else torch.as_tensor(np.asarray(x), dtype=torch.float32).to(dev).contiguous()
    nan = lambda shape: torch.full(tuple(shape), float("nan"), device=dev)
    chains = (w.batch, w.n_kv_heads, w.M, w.head_dim)
    out = dict(dq=nan(q.shape), dk=nan(k.shape), dv=nan(v.shape), d_cache0_k=nan(chains), d_cache0_v=nan(chains))
    dW = torch.zeros(cw.shape, dtype=torch.float32, device=dev)
    dB = None if cb is None else torch.zeros(cb.shape, dtype=torch.float32, device=dev)
    L = q.shape[2]
    ws = torch.empty(lb.lococo_sequence_backward_workspace_bytes(cfg, L, w.B), dtype=torch.uint8, device=dev)
    lb.lococo_sequence_backward(cfg, q.to(dev), k.to(dev), v.to(dev), w.B, cw.to(dev), None if cb is None else cb.to(dev),
                                cache, f32(r_o), f32(r_k), f32(r_v), out["dq"], out["dk"], out["dv"],
                                out["d_cache0_k"], out["d_cache0_v"], dW, dB, ws)
    torch.cuda.synchronize()
    assert torch.equal(cache.k, before[0]) and torch.equal(cache.v, before[1])      # the starting state is left alone
    assert (cache.len, cache.cur) == before[2:]
    got = {n: t.cpu().numpy() for n, t in out.items()}
    got["d_conv_w"], got["d_conv_b"] = dW.cpu().numpy(), None if dB is None else dB.cpu().numpy()
    return got


SCAN_CASES = [
    # fill, fill + compress boundary, compress...; a ragged last block; grouped heads
    dict(name="f32 from an empty cache, ragged tail", dtype="f32", batch=2, n_q_heads=4, n_kv_heads=2, head_dim=16,
         L=77, B=12, M=30, conv_width=5, len0=0, tol=3e-4),
    dict(name="f32 from a half-full cache, relu-sum, bias, per-head", dtype="f32", batch=1, n_q_heads=2, n_kv_heads=2,
         head_dim=8, L=60, B=10, M=24, conv_width=3, norm=1, bias_sigma=0.4, per_head_filters=True, len0=13,
         tol=3e-4),
    dict(name="f32 [K|V] filters, protected slots, no final gradient", dtype="f32", batch=1, n_q_heads=2,
         n_kv_heads=1, head_dim=16, L=64, B=16, M=16, conv_width=5, conv_in=1, len0=16, protect=True, final=False,
         tol=3e-4),
    dict(name="f32 one block", dtype="f32", batch=1, n_q_heads=1, n_kv_heads=1, head_dim=16, L=9, B=16, M=12,
         conv_width=3, len0=8, tol=3e-4),
    dict(name="f32 fills only", dtype="f32", batch=2, n_q_heads=2, n_kv_heads=1, head_dim=16, L=20, B=8, M=32,
         conv_width=3, len0=4, tol=3e-4),
    # bf16 storage, the fused compression kernel in the forward, the matrix-core contractions in the
    # backward.  The forward states are rounded to bf16 on both sides (the oracle rounds the exact value,
    # the kernel an fp32 one), so a few state entries differ by one bf16 step: the tolerance is that of
    # the storage type, not of the arithmetic.
    dict(name="bf16 head_dim 128 fused forward", dtype="bf16", batch=2, n_q_heads=4, n_kv_heads=2, head_dim=128,
         L=5 * 64 + 20, B=64, M=64, conv_width=15, len0=0, impl=0, tol=2e-3, state_round="bf16"),
    dict(name="bf16 head_dim 128 [K|V] width 21", dtype="bf16", batch=1, n_q_heads=2, n_kv_heads=2,
         head_dim=128, L=4 * 96, B=96, M=128, conv_width=21, conv_in=1, bias_sigma=0.4, len0=40, impl=0,
         tol=2e-3, state_round="bf16"),
    # relu + sum has a kink at every zero of a logit: where the two sides' states differ by a bf16 step and
    # a logit sits within that of zero, one side's rectifier passes it and the other's does not, and the
    # gradient jumps by that entry's whole share: the bound is a few such entries, not a rounding level
    dict(name="bf16 head_dim 128 [K|V] width 21 relu-sum", dtype="bf16", batch=1, n_q_heads=2, n_kv_heads=2,
         head_dim=128, L=4 * 96, B=96, M=128, conv_width=21, conv_in=1, norm=1, bias_sigma=0.4, len0=40, impl=0,
         tol=5e-2, state_round="bf16"),
]


@pytest.mark.parametrize("case", SCAN_CASES, ids=[c["name"] for c in SCAN_CASES])
def test_sequence_backward_matches_the_oracle_walked_in_reverse(case):
    c = dict(case)
    c.pop("name")
    len0, tol, impl = c.pop("len0"), c.pop("tol"), c.pop("impl", 1)
    use_protect, final, state_round = c.pop("protect", False), c.pop("final", True), c.pop("state_round", "none")
    w = inputs.Workload(name="bwdseq", seed=23, conv_gain=3.0, **c)
    rng = np.random.default_rng(17)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    if w.bias_sigma == 0.0:
        cb = None
    chains = (w.batch, w.n_kv_heads, w.M, w.head_dim)
    ck0 = torch.as_tensor(rng.standard_normal(chains) * 0.5).to(w.torch_dtype)
    cv0 = torch.as_tensor(rng.standard_normal(chains) * 0.5).to(w.torch_dtype)
    ck0[:, :, len0:], cv0[:, :, len0:] = 0, 0
    r_o = rng.standard_normal(q.shape)
    ln = min(w.M, len0 + w.L)
    r_k, r_v = rng.standard_normal(chains), rng.standard_normal(chains)
    r_k[:, :, ln:], r_v[:, :, ln:] = 0.0, 0.0
    protect = (rng.random(chains[:3]) < 0.2) if use_protect else None
    zero = np.zeros(chains)
    want = oracle_scan_backward(w, q, k, v, cw, cb, ck0.double().numpy(), cv0.double().numpy(), len0, r_o,
                                 r_k if final else zero, r_v if final else zero, protect, state_round)
    cfg = lb.config_for(w, impl=impl)
    got = _gpu_scan_backward(w, cfg, q, k, v, cw, cb, ck0, cv0, len0, r_o, r_k if final else None,
                             r_v if final else None, protect)
    errs = {}
    for n in ("dq", "dk", "dv", "d_cache0_k", "d_cache0_v", "d_conv_w", "d_conv_b"):
        if want[n] is None:
            continue
        if n == "d_conv_b" and w.norm == 0:
            continue
        if not np.abs(want[n]).max() > 0:
            assert not got[n].any(), n
            continue
        errs[n] = _rel(got[n], want[n])
        assert errs[n] < tol, (n, errs[n])
    assert not got["d_cache0_k"][:, :, len0:].any() and not got["d_cache0_v"][:, :, len0:].any()
    print(case["name"], {n: f"{e:.1e}" for n, e in errs.items()})


def test_sequence_backward_equals_the_steps_composed_by_hand_on_the_matrix_cores():
    """bf16, head_dim 128: the one-call scan backward against lococo_segment_step (forward, keeping the
    states) and lococo_segment_step_backward (reverse) called block by block: the same launches, so equal
    up to the order of the filter gradients' atomic sums.  Also: the filter gradient against a central
    difference of the ORACLE forward (bf16 inputs, exact arithmetic) along a random direction."""
    w = inputs.Workload(name="bwdseq_mfma", dtype="bf16", batch=1, n_q_heads=4, n_kv_heads=2, head_dim=128, L=4 * 48 + 16,
                        B=48, M=64, conv_width=15, seed=5, conv_gain=3.0)
    rng = np.random.default_rng(2)
    q, k, v = inputs.qkv(w)
    cw, _ = inputs.conv_filters(w)
    chains = (w.batch, w.n_kv_heads, w.M, w.head_dim)
    r_o, r_k, r_v = rng.standard_normal(q.shape), rng.standard_normal(chains), rng.standard_normal(chains)
    cfg = lb.config_for(w, impl=0)
    zeros = torch.zeros(chains, dtype=w.torch_dtype)
    got = _gpu_scan_backward(w, cfg, q, k, v, cw, None, zeros, zeros, 0, r_o, r_k, r_v, None)

    dev = "cuda"
    cache = lb.Cache(cfg, dev)
    qd, kd, vd, cwd = q.to(dev), k.to(dev), v.to(dev), cw.to(dev)
    ws = torch.empty(max(lb.lococo_workspace_bytes(cfg, w.B, w.B, 0), 256), dtype=torch.uint8, device=dev)
    starts = list(range(0, w.L, w.B))
    states = []
    for s0 in starts:
        states.append((cache.k.clone(), cache.v.clone(), cache.len))
        if s0 == starts[-1]:
            break                                # the state after the last block is not needed
        sl = slice(s0, s0 + w.B)
        o = torch.empty((w.batch, w.n_q_heads, w.B, w.head_dim), dtype=w.torch_dtype, device=dev)
        lb.lococo_segment_step(cfg, qd[:, :, sl], kd[:, :, sl], vd[:, :, sl], o, cwd, None, cache, ws)
    dW = torch.zeros(cw.shape, dtype=torch.float32, device=dev)
    gk, gv = r_k, r_v
    hand = dict(dq=np.zeros(q.shape, np.float32), dk=np.zeros(k.shape, np.float32), dv=np.zeros(k.shape, np.float32))
    for n in reversed(range(len(starts))):
        sl = slice(starts[n], starts[n] + w.B)
        ck, cv, m = states[n]
        step = _gpu_step_backward(w, cfg, q[:, :, sl].contiguous(), k[:, :, sl].contiguous(), v[:, :, sl].contiguous(),
                                  cw, None, ck.cpu(), cv.cpu(), m,
                                  r_o[:, :, sl], gk, gv, dW, None)
        hand["dq"][:, :, sl], hand["dk"][:, :, sl], hand["dv"][:, :, sl] = step["dq"], step["dk"], step["dv"]
        gk, gv = step["d_cache_k"], step["d_cache_v"]
    for n in ("dq", "dk", "dv"):
        assert _rel(got[n], hand[n]) < 1e-5, (n, _rel(got[n], hand[n]))
    assert _rel(got["d_conv_w"], dW.cpu().numpy()) < 1e-5
    assert not got["d_cache0_k"].any() and not got["d_cache0_v"].any()      # nothing was live at the start

    def loss(cw_):
        o, ck, cv, _ = orc.sequence_forward(q, k, v, cw_, None, B=w.B, M=w.M)
        return (o * r_o).sum() + (ck * r_k).sum() + (cv * r_v).sum()

    direction = rng.standard_normal(cw.shape)
    cw64, eps = cw.double().numpy(), 1e-5
    fd = (loss(cw64 + eps * direction) - loss(cw64 - eps * direction)) / (2 * eps)
    mine = float((got["d_conv_w"].astype(np.float64) * direction).sum())
    # the kernel's states are bf16, the oracle's loss is exact: agreement to the storage type's step
    assert abs(mine - fd) < 2e-2 * max(1.0, abs(fd)), (mine, fd)


def test_step_backward_on_a_full_size_block():
    """One compress step at the headline block and cache size (B = M = 512, head_dim 128, width 15) on two
    chains, every gradient against the oracle."""
    w = inputs.Workload(name="bwd512", dtype="bf16", batch=1, n_q_heads=2, n_kv_heads=2, head_dim=128, L=512, B=512,
                        M=512, conv_width=15, seed=31, conv_gain=3.0)
    rng = np.random.default_rng(6)
    q, k, v = inputs.qkv(w)
    cw, _ = inputs.conv_filters(w)
    chains = (w.batch, w.n_kv_heads, w.M, w.head_dim)
    ck = torch.as_tensor(rng.standard_normal(chains) * 0.5).to(w.torch_dtype)
    cv = torch.as_tensor(rng.standard_normal(chains) * 0.5).to(w.torch_dtype)
    d_o, gk, gv = rng.standard_normal(q.shape), rng.standard_normal(chains), rng.standard_normal(chains)
    want = orc.step_backward(q, k, v, ck, cv, w.M, cw, None, d_o, gk, gv, M=w.M)
    cfg = lb.config_for(w, impl=0)
    dW = torch.zeros(cw.shape, dtype=torch.float32, device="cuda")
    got = _gpu_step_backward(w, cfg, q, k, v, cw, None, ck, cv, w.M, d_o, gk, gv, dW, None)
    got["d_conv_w"] = dW.cpu().numpy()
    for n in ("dq", "dk", "dv", "d_cache_k", "d_cache_v", "d_conv_w"):
        assert _rel(got[n], want[n]) < 2e-4, (n, _rel(got[n], want[n]))


def test_sequence_backward_refusals():
    w = inputs.Workload(name="bwdseq_bad", dtype="f32", batch=1, n_q_heads=1, n_kv_heads=1, head_dim=16, L=32, B=8, M=8,
                        conv_width=3)
    cfg = lb.config_for(w, impl=1)
    q, k, v = (t.cuda() for t in inputs.qkv(w))
    cw, _ = inputs.conv_filters(w)
    cache = lb.Cache(cfg, "cuda")
    z = lambda *s: torch.zeros(s, device="cuda")
    g = dict(d_o=z(*q.shape), dq=z(*q.shape), dk=z(*k.shape), dv=z(*k.shape), ck=z(1, 1, 8, 16), cv=z(1, 1, 8, 16),
             dW=z(*cw.shape))
    need = lb.lococo_sequence_backward_workspace_bytes(cfg, w.L, w.B)
    small = torch.empty(need - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(lb.LococoError) as e:
        lb.lococo_sequence_backward(cfg, q, k, v, w.B, cw.cuda(), None, cache, g["d_o"], None, None, g["dq"], g["dk"],
                                    g["dv"], g["ck"], g["cv"], g["dW"], None, small)
    assert e.value.status == lb.LOCOCO_EWORKSPACE
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    with pytest.raises(lb.LococoError) as e:                 # the scan compresses: filters are needed
        lb.lococo_sequence_backward(cfg, q, k, v, w.B, None, None, cache, g["d_o"], None, None, g["dq"], g["dk"],
                                    g["dv"], g["ck"], g["cv"], g["dW"], None, ws)
    assert e.value.status == lb.LOCOCO_EINVAL
    cfg2 = lb.config_for(w.replace(norm=2), impl=1)
    with pytest.raises(lb.LococoError) as e:
        lb.lococo_sequence_backward(cfg2, q, k, v, w.B, cw.cuda(), None, cache, g["d_o"], None, None, g["dq"], g["dk"],
                                    g["dv"], g["ck"], g["cv"], g["dW"], None, ws)
    assert e.value.status == lb.LOCOCO_EUNSUPPORTED
