"""A seeded sweep over shapes and options of the bf16 / head_dim 128 path: every case draws its block
and cache sizes, head counts, filter width, normalisation, convolution input, filter sharing, bias,
sharpness, protected slots, initial cache occupancy, ragged tail and kernel family from its own
stream, runs the scan in all four schedules and compares the result with the oracle and the
schedules with each other (bit for bit).  A second sweep does the same for the shapes only the shape-agnostic
and unfused kernels take, with tracked attention and the entry point that allocates nothing."""
import numpy as np
import pytest
import torch

from oracle import lococo_oracle as orc
from paper_2406_05317_amd import binding as lb
from paper_2406_05317_amd import inputs
from parity_util import assert_close, compare_scan, gpu_forward, oracle_forward

pytestmark = pytest.mark.gpu
N_CASES = 56


def _draw(i):
    rng = np.random.default_rng(9000 + i)
    ch = lambda xs: xs[int(rng.integers(len(xs)))]
    M = ch([32, 64, 96, 128, 160, 192, 256, 320, 512])
    B = ch([1, 1, 5, 31, 32, 33, 64, 96, 100, 128, 160, 256, 300])
    norm = ch([0, 0, 1])
    if B > 4:
        n_blocks = min(-(-M // B) + int(rng.integers(0, 5)), 12)   # (rounding differences of the stored state add up along a scan)
        L = n_blocks * B + ch([0, 0, 1, int(rng.integers(1, B))])
        len0 = ch([0, 0, int(rng.integers(1, M + 1))])
    else:
        L = int(rng.integers(3, 10)) if B == 1 else int(rng.integers(2, 7)) * B + ch([0, 1, 2])
        len0 = ch([M, M - 1, M - 3, 0])
    if norm == 1:
        # The rectified sum amplifies a rounding difference of the state without bound where a row has almost no
        # positive logit, so under it a scan is compared up to the end of its first compression.
        plan = orc.plan(L, B, M, len0)
        first = np.nonzero(plan[:, 2] == 1)[0]
        if len(first):
            L = int(plan[first[0], 0] + plan[first[0], 1])
    Hkv, g, batch = ch([1, 2, 3, 4, 8]), ch([1, 1, 2, 4]), ch([1, 1, 2, 3])
    width, conv_in = ch([15, 21]), ch([0, 0, 1])
    per_head, bias = ch([False, False, True]), ch([0.0, 0.5])
    qg, cg = ch([(1, 1), (4, 3), (6, 6)])
    prot_kind = ch([None, None, "sinks", "scattered"])
    C = 128 * (2 if conv_in else 1)
    while batch * Hkv * (L // B + 1) * M * (M + B) * C * width > 4e10 and (batch > 1 or Hkv > 1):
        if batch > 1:
            batch -= 1
        else:
            Hkv = max(1, Hkv // 2)
    w = inputs.Workload(name=f"sweep{i}", dtype="bf16", batch=batch, n_q_heads=Hkv * g, n_kv_heads=Hkv, head_dim=128,
                        L=L, B=B, M=M, conv_width=width, conv_in=conv_in, norm=norm, per_head_filters=per_head,
                        bias_sigma=bias, qk_gain=qg, conv_gain=cg, seed=9000 + i)
    prot = None
    if prot_kind == "sinks":
        prot = np.zeros(M, bool)
        prot[:4] = True
    elif prot_kind == "scattered":
        prot = rng.random((batch, Hkv, M)) < 0.15
    return w, prot, len0, ch([True, False]), ch([0, 2]), ch([2, 3])


@pytest.mark.parametrize("i", range(N_CASES))
def test_drawn_case(i, options):
    w, prot, len0, pairs, impl, G = _draw(i)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    cache = oracle_cache = None
    if len0:
        gen = torch.Generator().manual_seed(i)
        ck = (torch.randn(w.batch, w.n_kv_heads, w.M, 128, generator=gen) / 11).to(torch.bfloat16)
        cv = (torch.randn(w.batch, w.n_kv_heads, w.M, 128, generator=gen) / 11).to(torch.bfloat16)
        ck[:, :, len0:] = 0
        cv[:, :, len0:] = 0
        cache = (ck, cv, len0)
        oracle_cache = (ck.double().numpy(), cv.double().numpy(), len0)
    what = f"{w} protect={None if prot is None else prot.shape} len0={len0} pairs={pairs} impl={impl} window={G}"
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16, protect=prot, cache=oracle_cache)
    if not pairs:
        options(lb.LOCOCO_OPT_NO_STEP_PIPELINE, 1)
    whole = gpu_forward(w, q, k, v, cw, cb, impl=impl, protect=prot, cache_init=cache, history=True)
    compare_scan(w, whole, want, what=what)
    for kw in (dict(history=G), dict(history=False), dict(step_by_step=True)):
        other = gpu_forward(w, q, k, v, cw, cb, impl=impl, protect=prot, cache_init=cache, **kw)
        ln = want[3]
        assert torch.equal(whole[0], other[0]), (kw, what)
        assert torch.equal(whole[1][:, :, :ln], other[1][:, :, :ln]), (kw, what)
        assert torch.equal(whole[2][:, :, :ln], other[2][:, :, :ln]), (kw, what)
        assert whole[3:] == other[3:], (kw, what)


def _draw_any_shape(i):
    """Shapes the fused kernels do not take (any head_dim, M, width; fp32 too), the rectifier on the convolution
    input, tracked attention and the entry point that allocates nothing."""
    rng = np.random.default_rng(29000 + i)
    ch = lambda xs: xs[int(rng.integers(len(xs)))]
    dtype, d = ch(["bf16", "f32"]), ch([8, 16, 32, 64, 128])
    M, B = ch([5, 12, 20, 33, 40, 64, 77, 96, 128, 160]), ch([1, 3, 6, 16, 24, 33, 40, 64, 100])
    norm = ch([0, 0, 1, 2])
    L = min(-(-M // B) + int(rng.integers(0, 4)), 10) * B + ch([0, 0, 1, int(rng.integers(0, B))])
    len0 = ch([0, 0, int(rng.integers(0, M + 1))])
    if norm:                                   # (see _draw: a sum near zero in the denominator)
        plan = orc.plan(L, B, M, len0)
        first = np.nonzero(plan[:, 2] == 1)[0]
        if len(first):
            L = int(plan[first[0], 0] + plan[first[0], 1])
    Hkv, g, batch = ch([1, 2, 3]), ch([1, 2, 4]), ch([1, 2])
    qg, cg = ch([(1, 1), (4, 3)])
    w = inputs.Workload(name=f"any{i}", dtype=dtype, batch=batch, n_q_heads=Hkv * g, n_kv_heads=Hkv, head_dim=d, L=L, B=B,
                        M=M, conv_width=ch([1, 3, 5, 7, 15, 21, 31, 61]), conv_in=ch([0, 0, 1]), norm=norm,
                        per_head_filters=ch([False, False, True]), bias_sigma=ch([0.0, 0.5]), qk_gain=qg, conv_gain=cg,
                        filter_abs=(norm == 2), seed=29000 + i)
    prot_kind = ch([None, None, "sinks", "scattered"])
    prot = None
    if prot_kind == "sinks":
        prot = np.zeros(M, bool)
        prot[:min(4, M)] = True
    elif prot_kind == "scattered":
        prot = rng.random((batch, Hkv, M)) < 0.15
    return w, prot, len0, ch([0, 1]), ch([False, True]), ch([False, True])


@pytest.mark.parametrize("i", range(40))
def test_drawn_case_of_any_shape(i):
    w, prot, len0, impl, track, noalloc = _draw_any_shape(i)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    if w.norm == 2:                            # signed row sums: keep them away from zero
        k, v = k.abs(), v.abs()
    cache = None
    ock = ocv = None
    if len0:
        gen = torch.Generator().manual_seed(i)
        ck = (torch.randn(w.batch, w.n_kv_heads, w.M, w.head_dim, generator=gen) / 3).to(w.torch_dtype)
        cv = (torch.randn(w.batch, w.n_kv_heads, w.M, w.head_dim, generator=gen) / 3).to(w.torch_dtype)
        if w.norm == 2:
            ck, cv = ck.abs(), cv.abs()
        ck[:, :, len0:] = 0
        cv[:, :, len0:] = 0
        cache, ock, ocv = (ck, cv, len0), ck.double().numpy(), cv.double().numpy()
    want_cs = np.zeros((w.batch, w.n_kv_heads, w.M))
    want = orc.sequence_forward(q, k, v, cw, cb, B=w.B, M=w.M, conv_in=w.conv_in, norm=w.norm, state_round=w.dtype,
                                cache_k=ock, cache_v=ocv, cache_len=len0, protect=prot,
                                attn_colsum=want_cs if track else None, nthreads=16)
    # fp32: 1e-5, and 1e-4 where a logit's own rounding is amplified (sharpened softmax; a rectified or signed sum
    # in the denominator)
    tol = 2e-2 if w.dtype == "bf16" else (1e-5 if w.qk_gain == 1 and w.norm == 0 else 1e-4)
    what = f"{w} protect={None if prot is None else prot.shape} len0={len0} impl={impl} track={track} noalloc={noalloc}"
    whole = gpu_forward(w, q, k, v, cw, cb, impl=impl, protect=prot, cache_init=cache, history=True)
    compare_scan(w, whole, want, tol=tol, what=what)
    ln = want[3]

    def same(other, tag):
        assert torch.equal(whole[0], other[0]), (tag, what)
        assert torch.equal(whole[1][:, :, :ln], other[1][:, :, :ln]), (tag, what)
        assert torch.equal(whole[2][:, :, :ln], other[2][:, :, :ln]), (tag, what)
        assert whole[3:] == tuple(other[3:]), (tag, what)

    for kw in (dict(history=2), dict(history=False), dict(step_by_step=True)):
        same(gpu_forward(w, q, k, v, cw, cb, impl=impl, protect=prot, cache_init=cache, **kw), kw)
    if not (track or noalloc):
        return
    cfg = lb.config_for(w, impl=impl)
    c = lb.Cache(cfg)
    c.set_protect(prot)
    if cache is not None:
        c.load(cache[0].cuda(), cache[1].cuda(), len0)
    if track:
        c.track_attention()
    qd, kd, vd, cwd = q.cuda(), k.cuda(), v.cuda(), cw.cuda().contiguous()
    cbd = None if cb is None else cb.cuda()
    od = torch.full_like(qd, float("nan"))
    if noalloc:
        for s in range(0, w.L, w.B):
            e = min(s + w.B, w.L)
            lb.lococo_segment_step_noalloc(cfg, qd[:, :, s:e], kd[:, :, s:e], vd[:, :, s:e], od[:, :, s:e], cwd, cbd, c)
    else:
        lb.lococo_sequence_forward(cfg, qd, kd, vd, od, cwd, cbd, c, w.B, lb.workspace(cfg, w.L, w.B, True))
    torch.cuda.synchronize()
    got = (od.cpu(), c.k.cpu(), c.v.cpu(), c.len, c.cur)
    if track:                                  # (asking for the sums may change the attention kernel: oracle, not bits)
        compare_scan(w, got, want, tol=tol, what="tracked " + what)
        if want_cs.max() > 0:
            assert_close(c.attn_colsum.cpu().double().numpy(), want_cs, max(tol, 2e-5), "attention column sums " + what)
    else:
        same(got, "no-allocation entry point")
