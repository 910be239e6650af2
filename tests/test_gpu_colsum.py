"""GPU parity of the accumulated attention scores per cache slot (what a heavy-hitter policy ranks
slots by) against the CPU oracle: prefill blocks on the shape-agnostic attention kernel and on the
MFMA one (row statistics + a column-sum pass), single tokens on the generation-stage kernel, and
the scan's outputs unchanged by asking for them."""
import numpy as np
import pytest
import torch

from paper_2406_05317_amd import inputs
from parity_util import TOL, assert_close, compare_scan, oracle_forward
from oracle import lococo_oracle as orc

pytestmark = pytest.mark.gpu

MFMA = 2


def _oracle(w, q, k, v, cw, cb, B, cache, colsum):
    ck = cv = None
    ln = 0
    if cache is not None:
        ck, cv, ln = cache
    return orc.sequence_forward(q, k, v, cw, cb, B=B, M=w.M, conv_in=w.conv_in, norm=w.norm, state_round=w.dtype,
                                cache_k=ck, cache_v=cv, cache_len=ln, attn_colsum=colsum, nthreads=16)


def _gpu_scan(w, q, k, v, cw, cb, impl, track=True):
    from paper_2406_05317_amd import binding as lb
    cfg = lb.config_for(w, impl=impl)
    qd, kd, vd, cwd = (t.cuda() for t in (q, k, v, cw))
    cbd = None if cb is None else cb.cuda()
    od = torch.full_like(qd, float("nan"))
    cache = lb.Cache(cfg)
    if track:
        cache.track_attention()
    ws = lb.workspace(cfg, w.L, w.B, True)
    lb.lococo_sequence_forward(cfg, qd, kd, vd, od, cwd, cbd, cache, w.B, ws)
    torch.cuda.synchronize()
    return (od.cpu(), cache.k.cpu(), cache.v.cpu(), cache.len, cache.cur), cache


@pytest.mark.parametrize("case", [
    dict(dtype="f32", batch=2, n_q_heads=4, n_kv_heads=2, head_dim=32, L=100, B=16, M=40, conv_width=5),
    dict(dtype="bf16", batch=1, n_q_heads=2, n_kv_heads=2, head_dim=64, L=160, B=32, M=64, conv_width=7),
    dict(dtype="bf16", batch=1, n_q_heads=8, n_kv_heads=4, head_dim=128, L=500, B=96, M=128, conv_width=15, impl=MFMA),
    # several 64-slot tiles, the last one ragged (M = 160); four query heads per kv head; ragged last block
    dict(dtype="bf16", batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, L=700, B=200, M=160, conv_width=15, impl=MFMA),
    # blocks shorter than a 32-row chunk
    dict(dtype="bf16", batch=1, n_q_heads=2, n_kv_heads=2, head_dim=128, L=150, B=20, M=64, conv_width=15, impl=MFMA),
])
def test_scan_accumulates_attention_per_slot(case):
    case = dict(case)
    impl = case.pop("impl", 1)
    w = inputs.Workload(name="colsum", seed=11, **case)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    want_cs = np.zeros((w.batch, w.n_kv_heads, w.M))
    want = _oracle(w, q, k, v, cw, cb, w.B, None, want_cs)
    got, cache = _gpu_scan(w, q, k, v, cw, cb, impl)
    compare_scan(w, got, want, what="colsum scan")
    assert want_cs.max() > 1.0                       # several query rows put real weight on the slots
    assert_close(cache.attn_colsum.cpu().double().numpy(), want_cs, max(TOL[w.dtype], 2e-5), "attention column sums")
    # the first block sees an empty cache: every row's probabilities sum to one, so the total
    # added per chain is (rows that saw a cache) * group minus what went to the block's own keys
    assert float(cache.attn_colsum.sum()) < (w.L - w.B) * w.n_q_heads * w.batch


def test_tracked_steps_one_by_one_on_the_mfma_kernels():
    """lococo_segment_step block by block with a step workspace (no history): the MFMA attention
    leaves its row statistics there and the column-sum pass follows; same sums as the oracle."""
    from paper_2406_05317_amd import binding as lb
    w = inputs.Workload(name="colsum", seed=15, dtype="bf16", batch=1, n_q_heads=4, n_kv_heads=2, head_dim=128,
                        L=600, B=128, M=192, conv_width=15)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    want_cs = np.zeros((w.batch, w.n_kv_heads, w.M))
    want = _oracle(w, q, k, v, cw, cb, w.B, None, want_cs)
    cfg = lb.config_for(w, impl=MFMA)
    qd, kd, vd, cwd = (t.cuda() for t in (q, k, v, cw))
    cbd = None if cb is None else cb.cuda()
    od = torch.full_like(qd, float("nan"))
    cache = lb.Cache(cfg)
    cache.track_attention()
    ws = lb.workspace(cfg, w.B, w.B, False)
    lb.lococo_timing_begin()
    for s0 in range(0, w.L, w.B):
        e = min(w.L, s0 + w.B)
        lb.lococo_segment_step(cfg, qd[:, :, s0:e], kd[:, :, s0:e], vd[:, :, s0:e], od[:, :, s0:e], cwd, cbd, cache, ws)
    torch.cuda.synchronize()
    ran = lb.lococo_timing_end()
    assert "attn_colsum" in ran and "attn_generic" not in ran, ran
    compare_scan(w, (od.cpu(), cache.k.cpu(), cache.v.cpu(), cache.len, cache.cur), want, what="tracked steps")
    assert_close(cache.attn_colsum.cpu().double().numpy(), want_cs, 2e-2, "attention column sums")


def test_tracking_leaves_the_scan_outputs_as_they_were():
    """The MFMA scan without tracking and with it (the attention kernel also writes its row
    statistics, a column-sum pass follows) give the same outputs."""
    w = inputs.Workload(name="colsum", seed=12, dtype="bf16", batch=1, n_q_heads=4, n_kv_heads=4, head_dim=128,
                        L=512, B=128, M=128, conv_width=15)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    a, _ = _gpu_scan(w, q, k, v, cw, cb, MFMA, track=False)
    b, _ = _gpu_scan(w, q, k, v, cw, cb, MFMA, track=True)
    assert_close(b[0].double().numpy(), a[0].double().numpy(), 2e-2, "O")
    assert torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])    # same compression kernels either way


@pytest.mark.parametrize("case", [
    dict(M=128, P=256, n_dec=12),
    dict(M=256, P=200, n_dec=70, n_q_heads=8, n_kv_heads=4),      # generation starts on a partly filled cache
])
def test_generation_steps_accumulate_attention_per_slot(case):
    """Prefill, then one token at a time on the generation-stage attention kernel; the accumulator
    runs on through both."""
    from paper_2406_05317_amd import binding as lb
    case = dict(case)
    P, n_dec = case.pop("P"), case.pop("n_dec")
    base = dict(name="colsum", seed=13, dtype="bf16", batch=2, n_q_heads=4, n_kv_heads=4, head_dim=128,
                L=P + n_dec, B=128, conv_width=15)
    base.update(case)
    w = inputs.Workload(**base)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    sl = lambda t, a, b: t[:, :, a:b]
    want_cs = np.zeros((w.batch, w.n_kv_heads, w.M))
    o1, ck, cv, ln = _oracle(w, sl(q, 0, P), sl(k, 0, P), sl(v, 0, P), cw, cb, w.B, None, want_cs)
    after_prefill = want_cs.copy()
    o2, ck, cv, ln = _oracle(w, sl(q, P, w.L), sl(k, P, w.L), sl(v, P, w.L), cw, cb, 1, (ck, cv, ln), want_cs)
    want = (np.concatenate([o1, o2], 2), ck, cv, ln)

    cfg = lb.config_for(w, impl=MFMA)
    qd, kd, vd, cwd, cbd = (t.cuda() for t in (q, k, v, cw, cb))
    od = torch.full_like(qd, float("nan"))
    cache = lb.Cache(cfg)
    cache.track_attention()
    lb.lococo_sequence_forward(cfg, sl(qd, 0, P), sl(kd, 0, P), sl(vd, 0, P), sl(od, 0, P), cwd, cbd, cache,
                               w.B, lb.workspace(cfg, P, w.B, True))
    torch.cuda.synchronize()
    assert_close(cache.attn_colsum.cpu().double().numpy(), after_prefill, 2e-2, "column sums after prefill")
    ws1 = lb.workspace(cfg, 1, 1, False)
    for t in range(P, w.L):
        lb.lococo_segment_step(cfg, sl(qd, t, t + 1), sl(kd, t, t + 1), sl(vd, t, t + 1), sl(od, t, t + 1),
                               cwd, cbd, cache, ws1)
    torch.cuda.synchronize()
    compare_scan(w, (od.cpu(), cache.k.cpu(), cache.v.cpu(), cache.len, cache.cur), want, what="generation")
    got_cs = cache.attn_colsum.cpu().double().numpy()
    assert_close(got_cs, want_cs, 2e-2, "column sums after generation")
    # what the generation steps alone added, against the oracle's increment
    assert_close(got_cs - after_prefill, want_cs - after_prefill, 3e-2, "generation-stage increment")


def test_large_memory_generation_step_takes_the_general_kernel():
    """A memory whose scores do not fit the generation kernel's LDS beside its partial states is
    attended by the shape-agnostic kernel when scores are tracked; same result."""
    from paper_2406_05317_amd import binding as lb
    w = inputs.Workload(name="colsum", seed=14, dtype="bf16", batch=1, n_q_heads=2, n_kv_heads=2, head_dim=128,
                        L=8192 + 2, B=8192, M=8192, conv_width=15)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    sl = lambda t, a, b: t[:, :, a:b]
    cfg = lb.config_for(w, impl=MFMA)
    qd, kd, vd, cwd, cbd = (t.cuda() for t in (q, k, v, cw, cb))
    # fill the cache with the first M tokens (no compression yet), then one generation step each way
    outs = []
    for track in (False, True):
        cache = lb.Cache(cfg)
        cache.load(sl(kd, 0, w.M), sl(vd, 0, w.M), w.M)
        if track:
            cache.track_attention()
        od = torch.full_like(sl(qd, w.M, w.M + 1), float("nan")).contiguous()
        lb.lococo_attn_only(cfg, sl(qd, w.M, w.M + 1), sl(kd, w.M, w.M + 1), sl(vd, w.M, w.M + 1), od, cache)
        torch.cuda.synchronize()
        outs.append(od.cpu().double().numpy())
    assert_close(outs[1], outs[0], 2e-2, "O")
    # one query row per head: each chain's slots receive (group) rows' probabilities, a little less than 1 each
    tot = cache.attn_colsum.sum(-1).cpu().numpy()
    assert np.all(tot > 0.9 * w.group) and np.all(tot <= w.group * (1 + 1e-5))
