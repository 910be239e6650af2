"""GPU parity at the full sizes of the measured configurations, in the launch
configuration bench.py times (one lococo_sequence_forward call with the
batched-attention workspace).  The oracle is too slow for every chain of the
large workloads, and chains are independent, so it recomputes sampled
(batch, kv-head) chains over the whole scan; all chains are additionally
checked on a truncated sequence in test_gpu_mfma.py-sized runs below."""
import numpy as np
import pytest
import torch

from oracle import lococo_oracle as orc
from paper_2406_05317_amd import inputs
from parity_util import TOL, assert_close, compare_scan, gpu_forward, oracle_forward, to_np

pytestmark = pytest.mark.gpu


def _check_sampled_chains(w, chains, L=None):
    L = L or w.L
    q, k, v = inputs.qkv(w, L)
    cw, cb = inputs.conv_filters(w)
    got = gpu_forward(w, q, k, v, cw, cb, history=True)
    o_g, ck_g, cv_g, ln_g, cur_g = got
    plan = orc.plan(L, w.B, w.M)
    assert ln_g == plan[-1, 4] and cur_g == plan[-1, 5]
    g = w.group
    tol = TOL[w.dtype]
    for (b, h) in chains:
        qs = q[b:b + 1, h * g:(h + 1) * g]
        want = orc.sequence_forward(qs, k[b:b + 1, h:h + 1], v[b:b + 1, h:h + 1],
                                    cw[h] if w.per_head_filters else cw,
                                    (cb[h] if w.per_head_filters else cb) if w.bias_sigma > 0 else None, B=w.B, M=w.M,
                                    conv_in=w.conv_in, norm=w.norm, state_round=w.dtype, nthreads=16)
        # the sampled chain regenerated on its own equals its slab of the full tensors
        qc, kc, vc = inputs.chain_inputs(w, b, h, L)
        assert torch.equal(qc, qs[0]) and torch.equal(kc, k[b, h]) and torch.equal(vc, v[b, h])
        e_o = assert_close(to_np(o_g[b, h * g:(h + 1) * g]), want[0][0], tol, f"{w.name} chain {b},{h} O")
        e_k = assert_close(to_np(ck_g[b, h]), want[1][0, 0], tol, f"{w.name} chain {b},{h} cache K")
        e_v = assert_close(to_np(cv_g[b, h]), want[2][0, 0], tol, f"{w.name} chain {b},{h} cache V")
        print(w.name, "chain", (b, h), "max-rel / l2-rel:", e_o, e_k, e_v)
    assert torch.isfinite(o_g.float()).all()
    return got


def test_cfg2_full_all_chains():
    w = inputs.CFG2
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16)
    got = gpu_forward(w, q, k, v, cw, cb, history=True)
    print(compare_scan(w, got, want, what="cfg2"))


def test_cfg3_full_sampled_chains():
    """The benchmark workload: 32 chains x 64 blocks; three chains recomputed by the oracle."""
    _check_sampled_chains(inputs.CFG3, [(0, 0), (0, 13), (0, 31)])


def test_cfg3_all_chains_first_blocks():
    w = inputs.CFG3
    L = 4 * w.B
    q, k, v = inputs.qkv(w, L)
    cw, cb = inputs.conv_filters(w)
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16)
    got = gpu_forward(w, q, k, v, cw, cb, history=True)
    compare_scan(w, got, want, what="cfg3 first 4 blocks")


def test_cfg3_shape_with_the_compressor_as_printed_sampled_chains():
    """The 32 K-token shape with Eq. 5 over [K | V], width 21, relu-sum and a bias (the fused kernel in two
    walks, two chains per workgroup, one launch), 16 blocks; two chains recomputed by the oracle."""
    w = inputs.CFG3.replace(name="cfg3_printed", conv_in=1, conv_width=21, norm=1, bias_sigma=0.5)
    _check_sampled_chains(w, [(0, 3), (0, 30)], L=16 * w.B)


def test_cfg4_full_sampled_chains():
    """All 512 chains over all 128 blocks (two fills + 126 compressions, four chains per workgroup in
    one launch, per-token scales) as the benchmark runs the workload; three chains recomputed by the
    oracle over the whole scan, where a bf16 state that is re-rounded at every step would show drift."""
    _check_sampled_chains(inputs.CFG4, [(0, 0), (7, 19), (15, 31)])


def test_cfg4_all_chains_first_blocks():
    """Every chain of the batch against the oracle on the first six blocks (two fills + four compressions)."""
    w = inputs.CFG4
    L = 6 * w.B
    q, k, v = inputs.qkv(w, L)
    cw, cb = inputs.conv_filters(w)
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16)
    got = gpu_forward(w, q, k, v, cw, cb, history=True)
    compare_scan(w, got, want, what="cfg4 first 6 blocks, all chains")


def test_cfg5_gqa_full_sampled_chains():
    _check_sampled_chains(inputs.CFG5, [(0, 0), (1, 7)])


def test_results_do_not_depend_on_the_schedule_at_full_size():
    w = inputs.CFG5
    L = 8 * w.B
    q, k, v = inputs.qkv(w, L)
    cw, cb = inputs.conv_filters(w)
    a = gpu_forward(w, q, k, v, cw, cb, history=True)
    b = gpu_forward(w, q, k, v, cw, cb, history=False)
    c = gpu_forward(w, q, k, v, cw, cb, history=True)
    for x, y, z in zip(a[:3], b[:3], c[:3]):
        assert torch.equal(x, y) and torch.equal(x, z)


def test_a_sequence_of_a_million_tokens():
    """2^20 tokens of two heads at the cfg3 block and cache sizes (2 048 blocks, 2 047 compressions): far past
    with the heads of the queries and of the output more than 2^31 elements apart.  The windowed and the step-by-step schedule
    agree bit for bit, a scan one block shorter is a prefix, and the last block matches the oracle run from
    the state the GPU itself reached a block earlier."""
    from paper_2406_05317_amd import binding as lb
    L, B, M = 1 << 20, 512, 512
    w = inputs.Workload(name="long", dtype="bf16", batch=1, n_q_heads=2, n_kv_heads=2, head_dim=128, L=L, B=B, M=M,
                        conv_width=15, seed=3, qk_gain=4, conv_gain=3)
    q, k, v = inputs.qkv(w)
    cw, _ = inputs.conv_filters(w)
    cfg = lb.config_for(w, impl=2)
    kd, vd, cwd = k.cuda(), v.cuda(), cw.cuda().contiguous()
    # the two query heads, and the two heads of the output, lie 2^31 + 2^27 elements apart in memory
    far = (1 << 31) + (1 << 27)
    q_store = torch.empty(far + L * 128, dtype=torch.bfloat16, device="cuda")
    o_store = torch.empty(far + L * 128, dtype=torch.bfloat16, device="cuda")
    qd = q_store.as_strided((1, 2, L, 128), (2 * far, far, 128, 1))
    qd.copy_(q)

    def run(Lx, history):
        od = o_store.as_strided((1, 2, Lx, 128), (2 * far, far, 128, 1))
        od.fill_(float("nan"))
        c = lb.Cache(cfg)
        ws = lb.workspace(cfg, Lx, B, history)
        lb.lococo_sequence_forward(cfg, qd[:, :, :Lx], kd[:, :, :Lx], vd[:, :, :Lx], od, cwd, None, c, B, ws)
        torch.cuda.synchronize()
        assert lb.lococo_scan_status(cfg, ws) == 0
        return od, c

    o_win, c_win = run(L, 8)
    o_win = o_win.clone()                  # (the runs share the output store)
    assert bool(torch.isfinite(o_win.float()).all())
    o_step, c_step = run(L, 0)
    assert torch.equal(o_win, o_step) and torch.equal(c_win.k, c_step.k) and torch.equal(c_win.v, c_step.v)
    o_pre, c_pre = run(L - B, 8)
    assert torch.equal(o_pre, o_win[:, :, :L - B])
    sl = slice(L - B, L)
    want = orc.sequence_forward(q[:, :, sl], k[:, :, sl], v[:, :, sl], cw, None, B=B, M=M, state_round="bf16",
                                cache_k=c_pre.k.cpu().double().numpy(), cache_v=c_pre.v.cpu().double().numpy(),
                                cache_len=M, nthreads=4)
    assert_close(to_np(o_win[:, :, sl].cpu()), want[0], TOL["bf16"], "O of the last block")
    assert_close(to_np(c_win.k.cpu()), want[1], TOL["bf16"], "final cache K")
    assert_close(to_np(c_win.v.cpu()), want[2], TOL["bf16"], "final cache V")
