"""GPU parity of the MFMA kernels (bf16, head_dim 128) against the CPU oracle:
shapes that span several tiles, ragged tails, partly filled caches, both
row-tile sizes of the fused compression kernel, and peaked softmaxes."""
import numpy as np
import pytest
import torch

from oracle import lococo_oracle as orc
from paper_2406_05317_amd import binding as lb
from paper_2406_05317_amd import inputs
from parity_util import compare_scan, gpu_forward, oracle_forward

pytestmark = pytest.mark.gpu
MFMA = 2


def _w(**kw):
    base = dict(name="mfma", dtype="bf16", batch=1, n_q_heads=4, n_kv_heads=4, head_dim=128, L=512,
                B=128, M=128, conv_width=15, seed=7)
    base.update(kw)
    return inputs.Workload(**base)


def _run(w, pairs=True, **kw):
    # (few chains: by default two workgroups per (chain, slot tile) take the steps in turn; pairs = False
    # runs the plain builds, one workgroup each)
    lb.lococo_debug_option(lb.LOCOCO_OPT_NO_STEP_PIPELINE, 0 if pairs else 1)
    try:
        return _run_inner(w, **kw)
    finally:
        lb.lococo_debug_option(lb.LOCOCO_OPT_NO_STEP_PIPELINE, 0)


def _run_inner(w, **kw):
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16)
    got = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, **kw)
    errs = compare_scan(w, got, want, what=w.name)
    plan = orc.plan(w.L, w.B, w.M)
    assert got[3] == plan[-1, 4] and got[4] == plan[-1, 5]
    return errs


@pytest.mark.parametrize("case", [
    dict(),                                               # cfg2-shaped, cut to 4 heads / 4 blocks
    dict(L=500),                                          # ragged last block (116 tokens)
    dict(M=64, B=64, L=320),                              # 32-row tiles, two row tiles per chain
    dict(M=96, B=80, L=400),                              # M % 64 != 0, T = 176 not a tile multiple
    dict(M=128, B=96, L=480),                             # partly filled cache at the first compress (m = 96)
    dict(M=128, B=160, L=480),                            # block larger than the cache
    dict(M=128, B=64, L=448, batch=2, n_q_heads=6, n_kv_heads=3),   # cfg4-shaped, two fills
    dict(M=256, B=256, L=1024, n_q_heads=8, n_kv_heads=2),          # cfg5-shaped GQA
    dict(M=512, B=512, L=2048, n_q_heads=2, n_kv_heads=2),          # cfg3-shaped chain
    dict(per_head_filters=True, bias_sigma=0.5),
    dict(tok_lognormal_sigma=0.5, seed=11),
])
@pytest.mark.parametrize("pairs", [True, False], ids=["pairs", "plain"])
def test_mfma_scan_matches_oracle(case, pairs):
    errs = _run(_w(**case), pairs=pairs)
    print(case, {k: (f"{e[0]:.2e}", f"{e[1]:.2e}") for k, e in errs.items()})


@pytest.mark.parametrize("case", [
    dict(L=640),
    dict(L=500),                                          # ragged last block
    dict(M=128, B=96, L=480),                             # partly filled cache at the first compress
    dict(M=128, B=64, L=448, batch=2, n_q_heads=6, n_kv_heads=3),   # two fills, GQA
    dict(M=256, B=256, L=1024, n_q_heads=8, n_kv_heads=2),
    dict(M=128, B=128, L=100),                            # nothing to compress: plain causal attention
])
def test_mfma_batched_attention_schedule(case):
    """Keeping every intermediate cache and running all blocks' attention as one
    launch gives the oracle's result, bit-identical to the step-by-step schedule."""
    w = _w(**case)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16)
    a = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True)
    compare_scan(w, a, want, what="history")
    b = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=False)
    for x, y in zip(a[:3], b[:3]):
        assert torch.equal(x[..., :a[3], :] if x.shape[2] == w.M else x,
                           y[..., :a[3], :] if y.shape[2] == w.M else y)
    assert a[3:] == b[3:]


@pytest.mark.parametrize("gains", [(0, 0), (1e-3, 1e-3), (30, 20), (100, 60), (300, 0), (0, 200)])
@pytest.mark.parametrize("shape", [
    dict(M=128, B=128), dict(M=512, B=512, n_q_heads=2, n_kv_heads=2),
    dict(M=96, B=80, n_kv_heads=2, conv_in=1, conv_width=21),
], ids=["32-slot tiles", "64-slot tiles", "[K|V] width 21"])
def test_extreme_magnitudes(gains, shape):
    """All-zero queries, keys and filters (uniform weights), and magnitudes that make both softmaxes
    one-hot in all but name (logits in the hundreds): one compression from the same state matches the
    oracle at the usual tolerance; a longer scan stays finite (there a selection may flip on a state
    that the two sides rounded differently, so it is not compared)."""
    one = (shape["M"] // shape["B"] + 1) * shape["B"]          # fills, then exactly one compression
    w = _w(qk_gain=gains[0], conv_gain=gains[1], bias_sigma=0.5, seed=5, L=one, **shape)
    _run(w, history=True)
    w4 = w.replace(L=w.M + 3 * w.B)
    q, k, v = inputs.qkv(w4)
    cw, cb = inputs.conv_filters(w4)
    got = gpu_forward(w4, q, k, v, cw, cb, impl=MFMA, history=True)
    assert all(bool(torch.isfinite(t.float()).all()) for t in got[:3])


@pytest.mark.parametrize("case", [
    dict(M=64, B=1, L=6, len0=64),                        # generation with known tokens, from a full cache
    dict(M=128, B=1, L=5, len0=126, n_q_heads=8, n_kv_heads=2),   # two fills, then compressions
    dict(M=128, B=64, L=4 * 64 + 1),                      # a ragged last block of one token
    dict(M=128, B=64, L=4 * 64 + 1, window=2),            # ... alone in the last window
])
def test_blocks_of_one_token_take_the_same_kernel_in_every_schedule(case):
    """Which kernel a block's attention runs on depends on the block alone: a block of one token goes to
    the generation-stage kernel whether the blocks are taken one by one or their attention is batched, so
    every schedule returns the same bits."""
    case = dict(case)
    len0, G = case.pop("len0", 0), case.pop("window", 3)
    w = _w(**case)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    cache = None
    if len0:
        gen = torch.Generator().manual_seed(3)
        ck = (torch.randn(w.batch, w.n_kv_heads, w.M, w.head_dim, generator=gen) / 11).to(torch.bfloat16)
        cv = (torch.randn(w.batch, w.n_kv_heads, w.M, w.head_dim, generator=gen) / 11).to(torch.bfloat16)
        ck[:, :, len0:] = 0
        cv[:, :, len0:] = 0
        cache = (ck, cv, len0)
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16,
                          cache=None if cache is None else (ck.double().numpy(), cv.double().numpy(), len0))
    lb.lococo_timing_begin()
    a = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True, cache_init=cache)
    ran = lb.lococo_timing_end()
    single = w.L if w.B == 1 else int(w.L % w.B == 1)
    assert ran.get("attn_decode", (0, 0))[0] == single, ran
    assert (ran.get("attn_mfma", (0, 0))[0] > 0) == (w.B > 1), ran
    assert a[3] == w.M
    compare_scan(w, a, want, what="blocks of one token")
    others = [gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=G, cache_init=cache),
              gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=False, cache_init=cache),
              gpu_forward(w, q, k, v, cw, cb, impl=MFMA, step_by_step=True, cache_init=cache)]
    for other in others:
        for x, y in zip(a[:3], other[:3]):
            assert torch.equal(x, y)
        assert a[3:] == other[3:]


@pytest.mark.parametrize("case", [
    dict(M=128, B=64, L=1024, window=3),                               # two fills; windows of 3: fills + one compress, then compress only
    dict(M=128, B=128, L=1500, window=2),                              # ragged last block in a window of its own
    dict(M=256, B=64, L=1024, window=2, n_q_heads=8, n_kv_heads=2),    # four fills: the fill phase spans two windows
    dict(M=128, B=96, L=960, window=4, batch=2, n_q_heads=6, n_kv_heads=3),   # partly filled cache at the first compress
    dict(M=512, B=512, L=4096, window=3, n_q_heads=16, n_kv_heads=16),        # 128 workgroups of 64 slots, 8 per chain
    dict(M=128, B=64, L=640, window=4, batch=12, n_q_heads=8, n_kv_heads=8),  # several chains per workgroup
    dict(M=128, B=128, L=900, window=3, conv_in=1, conv_width=21, norm=1, bias_sigma=0.5, impl=0),   # unfused MFMA path
    dict(M=128, B=128, L=896, window=5, protect_share=0.1, track=True),       # protected slots, attention per slot tracked
])
def test_windowed_history_equals_full_history_and_step_by_step(case, options):
    """A workspace that holds the states of a window of G blocks: the compression scan and the batched
    attention run window by window on a ring of G + 1 states.  Bit-identical to the whole-sequence
    history and to the step-by-step schedule; equal to the oracle."""
    case = dict(case)
    G, impl = case.pop("window"), case.pop("impl", MFMA)
    share, track = case.pop("protect_share", 0.0), case.pop("track", False)
    w = _w(**case)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    protect = (np.random.default_rng(5).random((w.batch, w.n_kv_heads, w.M)) < share) if share else None
    cfg = lb.config_for(w, impl=impl)
    full_bytes = lb.lococo_workspace_bytes(cfg, w.L, w.B, 1)
    win_bytes = lb.lococo_workspace_bytes(cfg, w.L, w.B, G)
    assert lb.lococo_workspace_bytes(cfg, w.L, w.B, 0) < win_bytes < full_bytes
    assert win_bytes == lb.lococo_workspace_bytes(cfg, 100 * w.L, w.B, G)      # independent of the sequence length
    lb.lococo_timing_begin()
    a = gpu_forward(w, q, k, v, cw, cb, impl=impl, history=G, protect=protect)
    ran = lb.lococo_timing_end()
    n_blocks = -(-w.L // w.B)
    assert ran["attn_mfma"][0] == -(-n_blocks // G), ran             # one attention launch per window
    b = gpu_forward(w, q, k, v, cw, cb, impl=impl, history=True, protect=protect)
    c = gpu_forward(w, q, k, v, cw, cb, impl=impl, history=False, protect=protect)
    options(lb.LOCOCO_OPT_SCAN_PER_STEP, 1)
    d = gpu_forward(w, q, k, v, cw, cb, impl=impl, history=G, protect=protect)
    for other in (b, c, d):
        for x, y in zip(a[:3], other[:3]):
            assert torch.equal(x, y)
        assert a[3:] == other[3:]
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16, protect=protect)
    compare_scan(w, a, want, what="windowed history")
    if track:
        # attention per slot, accumulated window by window (the row statistics of one window at a time)
        want_cs = np.zeros((w.batch, w.n_kv_heads, w.M))
        orc.sequence_forward(q, k, v, cw, cb, B=w.B, M=w.M, conv_in=w.conv_in, norm=w.norm, state_round=w.dtype,
                             protect=protect, attn_colsum=want_cs, nthreads=16)
        cache = lb.Cache(cfg)
        cache.set_protect(protect)
        cache.track_attention()
        od = torch.empty_like(q, device="cuda")
        lb.lococo_sequence_forward(cfg, q.cuda(), k.cuda(), v.cuda(), od, cw.cuda(), cb.cuda(), cache, w.B,
                                   lb.workspace(cfg, w.L, w.B, G))
        torch.cuda.synchronize()
        assert torch.equal(od.cpu(), a[0])
        from parity_util import assert_close
        assert_close(cache.attn_colsum.cpu().double().numpy(), want_cs, 2e-2, "attention column sums, windowed")


def test_mfma_resume_with_history_from_a_full_cache():
    """A scan continued from a full cache (no fill phase) under the batched schedule."""
    w = _w(L=768)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    full = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True)
    L1 = 384
    first = gpu_forward(w, q[:, :, :L1], k[:, :, :L1], v[:, :, :L1], cw, cb, impl=MFMA, history=True)
    rest = gpu_forward(w, q[:, :, L1:], k[:, :, L1:], v[:, :, L1:], cw, cb, impl=MFMA, history=True,
                       cache_init=(first[1], first[2], first[3]))
    assert torch.equal(torch.cat([first[0], rest[0]], 2), full[0])
    assert torch.equal(rest[1], full[1]) and torch.equal(rest[2], full[2]) and rest[3] == full[3]


def test_mfma_64_row_tiles():
    """Enough (chain, row tile) pairs to fill the chip, so the 64-row variant runs."""
    _run(_w(batch=2, n_q_heads=32, n_kv_heads=32, M=256, B=128, L=512))


@pytest.mark.parametrize("gains", [(6.0, 3.0), (10.0, 8.0)])
def test_mfma_sharpened(gains):
    """Peaked attention and mixing rows: wrong taps, seams or masks would show."""
    qk, cg = gains
    w = _w(qk_gain=qk, conv_gain=cg, L=640)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16)
    got = gpu_forward(w, q, k, v, cw, cb, impl=MFMA)
    compare_scan(w, got, want, what="sharp")
    lg = orc.conv_logits(k[0, 0, :256].double().numpy(), cw.double().numpy())
    assert orc.normalise(lg).max() > 0.05                 # far from the uniform 1/256


def test_mfma_step_by_step_equals_sequence_call():
    w = _w(L=640)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    a = gpu_forward(w, q, k, v, cw, cb, impl=MFMA)
    b = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, step_by_step=True)
    for x, y in zip(a[:3], b[:3]):
        assert torch.equal(x, y)
    assert a[3:] == b[3:]


def test_mfma_is_refused_for_shapes_it_does_not_take():
    from paper_2406_05317_amd import binding as lb
    for kw in (dict(head_dim=64), dict(conv_width=7), dict(conv_in=1, conv_width=9), dict(conv_width=61), dict(M=100),
               dict(dtype="f32")):
        w = _w(**kw)
        cfg = lb.config_for(w, impl=MFMA)
        with pytest.raises(lb.LococoError) as e:
            lb.lococo_workspace_bytes(cfg, w.L, w.B)
        assert e.value.status == lb.LOCOCO_EUNSUPPORTED
        # AUTO falls back to the shape-agnostic kernels
        assert lb.lococo_workspace_bytes(lb.config_for(w, impl=0), w.L, w.B) > 0


def test_one_launch_scan_equals_one_launch_per_step(options):
    """All compress steps of a scan in one launch (slot tiles of a chain handing the cache to each
    other inside the kernel) against one launch per step: bit-identical."""
    w = _w(M=256, B=128, L=1536, n_q_heads=8, n_kv_heads=8)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    a = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True)
    options(lb.LOCOCO_OPT_SCAN_PER_STEP, 1)
    b = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True)
    for x, y in zip(a[:3], b[:3]):
        assert torch.equal(x, y)
    assert a[3:] == b[3:]
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16)
    compare_scan(w, a, want, what="one-launch scan")


@pytest.mark.parametrize("case", [
    dict(M=256, B=128, L=1536, n_q_heads=8, n_kv_heads=8),            # 4 slot tiles per chain
    dict(M=512, B=512, L=4096, n_q_heads=16, n_kv_heads=16),          # 128 workgroups, 8 tiles per chain
    dict(M=128, B=96, L=1000, n_q_heads=4, n_kv_heads=2, batch=2),    # ragged blocks, grouped heads
])
def test_chain_meeting_through_the_shared_l2_equals_the_device_scope_one(case, options):
    """Between the steps of the one-launch scan the slot tiles of a chain meet without writing the
    L2 back when they find themselves on one XCD; with the debug option LOCOCO_OPT_CHAIN_SYNC_DEVICE they always use
    device-scope release / acquire.  Same kernel arithmetic either way: bit-identical results,
    several runs each (a stale read would show as a difference)."""
    w = _w(**case)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    options(lb.LOCOCO_OPT_CHAIN_SYNC_DEVICE, 1)
    ref = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True)
    options(lb.LOCOCO_OPT_CHAIN_SYNC_DEVICE, 0)
    for _ in range(4):
        got = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True)
        for x, y in zip(got[:3], ref[:3]):
            assert torch.equal(x, y)
        assert got[3:] == ref[3:]
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16)
    compare_scan(w, ref, want, what="device-scope chain meeting")


@pytest.mark.parametrize("case", [
    # 96 chains x 4 slot tiles of 32 for 256 compute units: 64 workgroups per tile, one or two chains each
    dict(batch=12, n_q_heads=8, n_kv_heads=8, M=128, B=64, L=448),
    # 320 chains x 2 slot tiles of 64, filters per head: 128 workgroups per tile, two or three chains each
    dict(batch=5, n_q_heads=64, n_kv_heads=64, M=128, B=64, L=384, per_head_filters=True, bias_sigma=0.5),
    # grouped query heads, ragged last block, partly filled cache at the first compress step
    dict(batch=40, n_q_heads=8, n_kv_heads=4, M=64, B=48, L=300, tok_lognormal_sigma=0.5),
    # width 21 and relu-sum (32-slot tiles only): 40 chains x 8 tiles on 256 compute units
    dict(batch=5, n_q_heads=8, n_kv_heads=8, M=256, B=96, L=640, conv_width=21, norm=1, bias_sigma=0.5),
    # protected slots, different ones in every chain, with several chains per workgroup, 64-slot tiles
    dict(batch=24, n_q_heads=8, n_kv_heads=8, M=128, B=64, L=384, protect_share=0.1),
])
def test_one_launch_scan_with_several_chains_per_workgroup(case, options):
    """More (chain, slot tile) pairs than compute units: the one-launch scan gives every workgroup
    several chains of one slot tile.  Bit-identical to one launch per step, with either form of the
    chain meeting, and equal to the oracle."""
    case = dict(case)
    share = case.pop("protect_share", 0.0)
    w = _w(**case)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    protect = (np.random.default_rng(5).random((w.batch, w.n_kv_heads, w.M)) < share) if share else None
    a = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True, protect=protect)
    options(lb.LOCOCO_OPT_CHAIN_SYNC_DEVICE, 1)
    c = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True, protect=protect)
    options(lb.LOCOCO_OPT_CHAIN_SYNC_DEVICE, 0)
    options(lb.LOCOCO_OPT_SCAN_PER_STEP, 1)
    b = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True, protect=protect)
    for other in (b, c):
        for x, y in zip(a[:3], other[:3]):
            assert torch.equal(x, y)
        assert a[3:] == other[3:]
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16, protect=protect)
    compare_scan(w, a, want, what="several chains per workgroup")


@pytest.mark.parametrize("case", [
    dict(conv_in=1, conv_width=21, norm=1, bias_sigma=0.5, L=640),              # the compressor as the paper prints it
    dict(conv_in=1, conv_width=15, M=256, B=128, L=1024, n_q_heads=8, n_kv_heads=2, per_head_filters=True),
    dict(conv_width=7, L=500),                                                   # a width the fused kernel is not built for; ragged last block
    dict(conv_width=31, M=100, B=60, L=400),                                     # M not a multiple of 32, widest filter
    dict(conv_in=1, conv_width=3, M=64, B=48, L=300, batch=3, n_q_heads=4, n_kv_heads=2, tok_lognormal_sigma=0.5),
    dict(conv_in=1, conv_width=21, conv_gain=6.0, qk_gain=6.0, L=640),           # peaked rows
    dict(conv_in=1, conv_width=21, L=512, protect_share=0.15),                   # protected slots
    dict(conv_in=1, conv_width=31, M=384, B=200, L=1000, n_q_heads=2, n_kv_heads=2, bias_sigma=0.5),   # 256-slot tiles, the second half empty
    dict(conv_in=1, conv_width=21, norm=1, M=512, B=256, L=1536, n_q_heads=2, n_kv_heads=1),      # two full 256-slot tiles
    dict(conv_width=9, M=320, B=128, L=900, n_q_heads=2, n_kv_heads=2),                          # keys-only filters on the 256-slot tiles
    dict(conv_in=1, conv_width=21, norm=1, batch=4, n_q_heads=32, n_kv_heads=32, L=384),          # enough chains for 128-slot tiles, [K | V]
    dict(conv_width=7, batch=4, n_q_heads=32, n_kv_heads=32, L=384),                             # the same, keys only
])
def test_unfused_mfma_path_for_shapes_the_fused_kernel_does_not_take(case, options):
    """impl = AUTO with bf16 / head_dim 128 and a compressor the fused kernel is not built for
    ([K | V] input, other widths, odd M): MFMA attention, MFMA logits and MFMA fusion around the
    shape-agnostic normalisation.  Equal to the oracle; the timing rows say which kernels ran.
    Then every tile shape of the logits kernel, forced from the host: each equal to the oracle,
    the 64- and 128-slot tiles equal to each other bit for bit."""
    from paper_2406_05317_amd import binding as lb
    case = dict(case)
    share = case.pop("protect_share", 0.0)
    w = _w(**case)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    protect = (np.random.default_rng(6).random((w.batch, w.n_kv_heads, w.M)) < share) if share else None
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16, protect=protect)
    options(lb.LOCOCO_OPT_UNFUSED_KV, 1)       # (the fused kernel takes [K | V] filters of width 15 and 21: tested below)
    lb.lococo_timing_begin()
    got = gpu_forward(w, q, k, v, cw, cb, impl=0, history=True, protect=protect)
    ran = lb.lococo_timing_end()
    assert "conv_logits_mfma" in ran and "attn_mfma" in ran and "mix_mfma" in ran, ran
    assert "conv_logits_generic" not in ran and "attn_generic" not in ran, ran
    compare_scan(w, got, want, what="unfused MFMA path")
    # block by block through lococo_segment_step: the same kernels, the same bits
    again = gpu_forward(w, q, k, v, cw, cb, impl=0, step_by_step=True, protect=protect)
    for x, y in zip(got[:3], again[:3]):
        assert torch.equal(x, y)
    by_shape = {}
    for shape in ("64", "128", "256"):
        options(lb.LOCOCO_OPT_LOGITS_TILES, int(shape))
        by_shape[shape] = gpu_forward(w, q, k, v, cw, cb, impl=0, history=True, protect=protect)
        compare_scan(w, by_shape[shape], want, what="logits tiles of %s slots" % shape)
    options(lb.LOCOCO_OPT_LOGITS_TILES, 0)
    for x, y in zip(by_shape["64"][:3], by_shape["128"][:3]):
        assert torch.equal(x, y)


KV_CASES = [
    dict(conv_width=21, norm=1, bias_sigma=0.5, L=640),                             # the compressor as the paper prints it
    dict(conv_width=21, L=640),                                                     # the same filters under the softmax
    dict(conv_width=21, conv_gain=6.0, qk_gain=6.0, L=640),                         # peaked rows
    dict(conv_width=15, M=256, B=128, L=1000, n_q_heads=8, n_kv_heads=2, per_head_filters=True, bias_sigma=0.3, norm=1, split=2),
    dict(conv_width=21, M=256, B=128, L=640, n_q_heads=20, n_kv_heads=20),          # 160 pairs: one workgroup each, no split
    dict(conv_width=21, M=128, B=96, L=500),                                        # partly filled cache at the first compress, ragged last block
    dict(conv_width=21, M=96, B=200, L=640),                                        # block longer than the cache, T = 296 not a tile multiple
    dict(conv_width=21, L=512, protect_share=0.15),                                 # protected slots
    dict(conv_width=15, norm=1, L=512, protect_share=0.3, bias_sigma=0.5),
    dict(conv_width=21, norm=1, batch=4, n_q_heads=32, n_kv_heads=32, L=512),       # more (chain, tile) pairs than compute units: several chains per workgroup
    dict(conv_width=21, M=256, B=256, L=1024, n_q_heads=4, n_kv_heads=2, split=2),  # few pairs: the positions of a step shared out
    dict(conv_width=15, M=512, B=512, L=2048, n_q_heads=2, n_kv_heads=1, norm=1, split=4, protect_share=0.1),
    dict(conv_width=21, M=512, B=512, L=2048, n_q_heads=8, n_kv_heads=8, tok_lognormal_sigma=0.5, split=2),   # the 32 K-token shape's chains, 8 of them
]


@pytest.mark.parametrize("case", KV_CASES, ids=[str(i) for i in range(len(KV_CASES))])
def test_fused_kernel_with_filters_over_keys_and_values(case, options):
    """Eq. 5 over [K | V] (256 channels) on the fused kernel: two walks per step, the key half of the filters
    first (summed logits through the workspace), then the value half with softmax and mixing.  Against the
    oracle; the one-launch scan, one launch per step and lococo_segment_step give the same bits; the
    unfused MFMA path (another order of the fp32 sums) meets the same tolerance."""
    case = dict(case)
    share, split = case.pop("protect_share", 0.0), case.pop("split", 1)
    w = _w(conv_in=1, **case)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    protect = (np.random.default_rng(6).random((w.batch, w.n_kv_heads, w.M)) < share) if share else None
    cfg = lb.config_for(w, impl=MFMA)
    pairs = w.batch * w.n_kv_heads * (w.M // 32)
    options(lb.LOCOCO_OPT_NO_STEP_PIPELINE, 1)       # first without the pairs of workgroups over the steps
    info = lb.lococo_describe_path(cfg, w.B)
    assert info["path"] == 1 and info["tile_slots"] == 32 and info["position_split"] == split, info
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16, protect=protect)
    if 2 * pairs <= info["compute_units"]:
        plain = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True, protect=protect)
        compare_scan(w, plain, want, what="fused [K | V], one workgroup per pair or a position split")
        options(lb.LOCOCO_OPT_NO_STEP_PIPELINE, 0)
        assert lb.lococo_describe_path(cfg, w.B)["step_pipeline"] == 2
    lb.lococo_timing_begin()
    a = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True, protect=protect)
    ran = lb.lococo_timing_end()
    assert "compress_mfma" in ran and "conv_logits_mfma" not in ran and "mix_mfma" not in ran, ran
    errs = compare_scan(w, a, want, what="fused [K | V]")
    print(case, {n: (f"{e[0]:.2e}", f"{e[1]:.2e}") for n, e in errs.items()})
    options(lb.LOCOCO_OPT_SCAN_PER_STEP, 1)
    b = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True, protect=protect)
    options(lb.LOCOCO_OPT_SCAN_PER_STEP, 0)
    c = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, step_by_step=True, protect=protect)
    d = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=2, protect=protect)
    for other in (b, c, d):
        for x, y in zip(a[:3], other[:3]):
            assert torch.equal(x, y)
        assert a[3:] == other[3:]
    options(lb.LOCOCO_OPT_UNFUSED_KV, 1)
    u = gpu_forward(w, q, k, v, cw, cb, impl=0, history=True, protect=protect)
    compare_scan(w, u, want, what="unfused [K | V]")


def test_a_chain_wait_that_gives_up_is_reported(options):
    """Forced from the host: with no polls allowed, the first slot tile to finish a step cannot wait
    for its chain, leaves the kernel, and the status word says so.  Every workgroup still exits."""
    from paper_2406_05317_amd import binding as lb
    w = _w(M=256, B=128, L=1024, n_q_heads=4, n_kv_heads=4)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    cfg = lb.config_for(w, impl=MFMA)
    ws = lb.workspace(cfg, w.L, w.B, True)
    cache = lb.Cache(cfg)
    o = torch.empty_like(q, device="cuda")
    options(lb.LOCOCO_OPT_SPIN_LIMIT, -1)
    lb.lococo_sequence_forward(cfg, q.cuda(), k.cuda(), v.cuda(), o, cw.cuda(), cb.cuda(), cache, w.B, ws)
    assert lb.lococo_scan_status(cfg, ws) == 1
    options(lb.LOCOCO_OPT_SPIN_LIMIT, 0)
    cache = lb.Cache(cfg)
    lb.lococo_sequence_forward(cfg, q.cuda(), k.cuda(), v.cuda(), o, cw.cuda(), cb.cuda(), cache, w.B, ws)
    assert lb.lococo_scan_status(cfg, ws) == 0           # the word is cleared by the next call


@pytest.mark.parametrize("case", [
    dict(M=128, P=256, n_dec=16),                          # 32-row tiles, T = 129 = 4 tiles + one position
    dict(M=256, P=512, n_dec=12, n_q_heads=8, n_kv_heads=4),    # grouped query heads
    dict(M=128, P=100, n_dec=40),                          # decode starts with a partly filled cache: 28 fills, 12 compress steps
    # the unfused MFMA path: T = M + 1 is odd, so the logits rows are padded to a multiple of 4
    dict(M=128, P=256, n_dec=14, conv_in=1, conv_width=21, norm=1, bias_sigma=0.5, impl=0),
    dict(M=96, P=200, n_dec=10, conv_width=9, n_q_heads=8, n_kv_heads=2, impl=0),
])
def test_mfma_decode_after_prefill(case):
    """Generation stage: prefill in blocks, then one token at a time (segment steps with B = 1,
    T = M + 1), against the oracle run with the same two block sizes.  Every decode step rewrites
    the whole cache in bf16, so the two free-running states drift apart by a rounding step per
    token; the run is kept short enough for the contract tolerance and the per-step test below
    covers long generations."""
    from paper_2406_05317_amd import binding as lb
    case = dict(case)
    P, n_dec, impl = case.pop("P"), case.pop("n_dec"), case.pop("impl", MFMA)
    w = _w(L=P + n_dec, B=128, **case)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    sl = lambda t, a, b: t[:, :, a:b]
    o1, ck, cv, ln = oracle_forward(w, sl(q, 0, P), sl(k, 0, P), sl(v, 0, P), cw, cb, nthreads=16)
    o2, ck, cv, ln = oracle_forward(w, sl(q, P, w.L), sl(k, P, w.L), sl(v, P, w.L), cw, cb, B=1,
                                    cache=(ck, cv, ln), nthreads=16)
    want = (np.concatenate([o1, o2], 2), ck, cv, ln)

    cfg = lb.config_for(w, impl=impl)
    qd, kd, vd, cwd = (t.cuda() for t in (q, k, v, cw))
    cbd = None if cb is None else cb.cuda()
    od = torch.full_like(qd, float("nan"))
    cache = lb.Cache(cfg)
    ws = lb.workspace(cfg, P, w.B, True)
    lb.lococo_sequence_forward(cfg, sl(qd, 0, P), sl(kd, 0, P), sl(vd, 0, P), sl(od, 0, P), cwd, cbd, cache,
                               w.B, ws)
    ws1 = lb.workspace(cfg, 1, 1, False)
    for t in range(P, w.L):
        lb.lococo_segment_step(cfg, sl(qd, t, t + 1), sl(kd, t, t + 1), sl(vd, t, t + 1), sl(od, t, t + 1),
                               cwd, cbd, cache, ws1)
    torch.cuda.synchronize()
    got = (od.cpu(), cache.k.cpu(), cache.v.cpu(), cache.len, cache.cur)
    errs = compare_scan(w, got, want, what="decode")
    print(case, {k_: (f"{e[0]:.2e}", f"{e[1]:.2e}") for k_, e in errs.items()})


def test_mfma_decode_steps_from_the_oracle_state():
    """A long generation checked step by step: before every token the GPU cache is set to the
    oracle's current state, so each B = 1 step is compared on its own (no drift between the two
    recursions) over 96 tokens."""
    from paper_2406_05317_amd import binding as lb
    w = _w(M=128, L=128 + 96, B=128)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    sl = lambda t, a, b: t[:, :, a:b]
    _, ck, cv, ln = oracle_forward(w, sl(q, 0, 128), sl(k, 0, 128), sl(v, 0, 128), cw, cb, nthreads=16)
    cfg = lb.config_for(w, impl=MFMA)
    qd, kd, vd, cwd, cbd = (t.cuda() for t in (q, k, v, cw, cb))
    ws1 = lb.workspace(cfg, 1, 1, False)
    worst = 0.0
    for t in range(128, w.L):
        cache = lb.Cache(cfg)
        cache.load(torch.as_tensor(ck).to("cuda", w.torch_dtype), torch.as_tensor(cv).to("cuda", w.torch_dtype), ln)
        od = torch.full_like(sl(qd, t, t + 1), float("nan")).contiguous()
        lb.lococo_segment_step(cfg, sl(qd, t, t + 1), sl(kd, t, t + 1), sl(vd, t, t + 1), od, cwd, cbd, cache, ws1)
        o, ck, cv, ln = oracle_forward(w, sl(q, t, t + 1), sl(k, t, t + 1), sl(v, t, t + 1), cw, cb, B=1,
                                       cache=(ck, cv, ln), nthreads=4)
        errs = compare_scan(w, (od.cpu(), cache.k.cpu(), cache.v.cpu(), cache.len, cache.cur), (o, ck, cv, ln),
                            what=f"decode step {t}")
        worst = max(worst, max(e[0] for e in errs.values()))
    print("worst per-step max-rel", f"{worst:.2e}")
    assert worst < 1e-2


def test_prepared_filters_give_the_same_steps():
    """lococo_prepare_filters once + LOCOCO_FLAG_FILTERS_PREPARED on every step is bit-identical
    to letting every step repack the filter bank itself."""
    from paper_2406_05317_amd import binding as lb
    w = _w(M=128, L=128 + 8, B=128)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    qd, kd, vd, cwd, cbd = (t.cuda() for t in (q, k, v, cw, cb))
    sl = lambda t, a, b: t[:, :, a:b]
    outs = []
    for prepared in (False, True):
        cfg = lb.config_for(w, impl=MFMA)
        cache = lb.Cache(cfg)
        od = torch.full_like(qd, float("nan"))
        ws = lb.workspace(cfg, 128, 128, False)
        lb.lococo_segment_step(cfg, sl(qd, 0, 128), sl(kd, 0, 128), sl(vd, 0, 128), sl(od, 0, 128), cwd, cbd, cache, ws)
        if prepared:
            ws.zero_()                                       # nothing left over from the step above
            lb.lococo_prepare_filters(cfg, cwd, ws)
            cfg.flags |= lb.LOCOCO_FLAG_FILTERS_PREPARED
        for t in range(128, w.L):
            lb.lococo_segment_step(cfg, sl(qd, t, t + 1), sl(kd, t, t + 1), sl(vd, t, t + 1), sl(od, t, t + 1),
                                   cwd, cbd, cache, ws)
        torch.cuda.synchronize()
        outs.append((od.cpu(), cache.k.cpu(), cache.v.cpu(), cache.len, cache.cur))
    for x, y in zip(outs[0][:3], outs[1][:3]):
        assert torch.equal(x, y)
    assert outs[0][3:] == outs[1][3:]


@pytest.mark.parametrize("case", [
    dict(conv_width=21),                                            # the paper's default width
    dict(conv_width=21, L=500),                                     # ragged last block
    dict(conv_width=21, M=96, B=80, L=400),                         # T = 176 not a tile multiple, M % 64 != 0
    dict(conv_width=21, M=256, B=256, L=1024, n_q_heads=8, n_kv_heads=2, per_head_filters=True),
    dict(norm=1, bias_sigma=0.5),                                   # relu-sum normalisation (Eq. 6 as printed)
    dict(norm=1, bias_sigma=0.5, L=500),
    dict(norm=1, conv_width=21, bias_sigma=0.5, M=128, B=160, L=480),
    dict(norm=1, bias_sigma=0.5, batch=2, n_q_heads=32, n_kv_heads=32, M=256, B=128, L=512),   # 64-row tiles
    dict(norm=1, conv_gain=6.0, bias_sigma=1.0, L=640),             # peaked, many exactly-zero weights
])
def test_mfma_paper_literal_variants(case):
    """Width 21 and the relu-sum normalisation on the MFMA kernels, with the history schedule (one-launch
    scan where it fits) and without."""
    w = _w(**case)
    for history in (False, True):
        errs = _run(w, history=history)
    print(case, {k: (f"{e[0]:.2e}", f"{e[1]:.2e}") for k, e in errs.items()})


def test_decode_steps_replayed_from_a_hip_graph():
    """Two generation steps (the cache ping-pong returns to its first buffer after two) captured in
    a HIP graph and replayed several times with fresh tokens in the static input buffers, with
    eager work and synchronisations between the replays: every replay equals the eager steps."""
    from paper_2406_05317_amd import binding as lb
    w = _w(M=128, L=128 + 12, B=128)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    qd, kd, vd, cwd, cbd = (t.cuda() for t in (q, k, v, cw, cb))
    sl = lambda t, a, b: t[:, :, a:b]

    def prefill(cfg):
        cache = lb.Cache(cfg)
        o = torch.empty_like(sl(qd, 0, 128))
        lb.lococo_segment_step(cfg, sl(qd, 0, 128), sl(kd, 0, 128), sl(vd, 0, 128), o, cwd, cbd, cache,
                               lb.workspace(cfg, 128, 128, False))
        return cache

    # eager reference
    cfg = lb.config_for(w, impl=MFMA)
    cache = prefill(cfg)
    ws = lb.workspace(cfg, 1, 1, False)
    lb.lococo_prepare_filters(cfg, cwd, ws)
    cfg.flags |= lb.LOCOCO_FLAG_FILTERS_PREPARED
    want = torch.empty_like(sl(qd, 128, w.L))
    for t in range(128, w.L):
        lb.lococo_segment_step(cfg, sl(qd, t, t + 1), sl(kd, t, t + 1), sl(vd, t, t + 1), sl(want, t - 128, t - 127),
                               cwd, cbd, cache, ws)
    torch.cuda.synchronize()
    want_k, want_v = cache.k.clone(), cache.v.clone()

    # graph: static two-token buffers
    cache = prefill(cfg)
    cur0 = cache.cur
    sq, sk, sv = (torch.zeros_like(sl(x, 0, 2)).contiguous() for x in (qd, kd, vd))
    so = torch.zeros_like(sq)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            for i in range(2):
                lb.lococo_segment_step(cfg, sl(sq, i, i + 1), sl(sk, i, i + 1), sl(sv, i, i + 1), sl(so, i, i + 1),
                                       cwd, cbd, cache, ws)
    assert cache.cur == cur0                      # two steps: the live buffer is the first one again
    cache.c.len = w.M
    got = torch.empty_like(want)
    for t in range(128, w.L, 2):
        sq.copy_(sl(qd, t, t + 2)); sk.copy_(sl(kd, t, t + 2)); sv.copy_(sl(vd, t, t + 2))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got[:, :, t - 128:t - 126] = so             # eager work between replays
    assert torch.equal(got, want)
    assert torch.equal(cache.k, want_k) and torch.equal(cache.v, want_v)


@pytest.mark.parametrize("history", [True, 2, False], ids=["whole-sequence history", "windows of two blocks", "step by step"])
def test_a_whole_scan_replayed_from_a_hip_graph(history):
    """lococo_sequence_forward captured once into a HIP graph (the one-launch compression scan, the batched
    attention, the copy of the final state: kernels only, no memset node) and replayed several times on fresh
    inputs in the static buffers, with eager work and synchronisations between the replays: every replay
    equals the eager call on the same inputs, bit for bit."""
    w = _w(M=128, B=128, L=128 * 5 + 40, n_q_heads=8, n_kv_heads=4, bias_sigma=0.5)
    cfg = lb.config_for(w, impl=MFMA)
    cw, cb = inputs.conv_filters(w)
    cwd, cbd = cw.cuda().contiguous(), cb.cuda()
    ws = lb.workspace(cfg, w.L, w.B, history)

    def data(seed):
        q, k, v = inputs.qkv(w.replace(seed=seed))
        return q.cuda(), k.cuda(), v.cuda()

    def eager(q, k, v):
        o = torch.full_like(q, float("nan"))
        cache = lb.Cache(cfg)
        lb.lococo_sequence_forward(cfg, q, k, v, o, cwd, cbd, cache, w.B, ws)
        torch.cuda.synchronize()
        return o, cache.k.clone(), cache.v.clone(), cache.len, cache.cur

    sq, sk, sv = data(100)
    so = torch.zeros_like(sq)
    cache = lb.Cache(cfg)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            lb.lococo_sequence_forward(cfg, sq, sk, sv, so, cwd, cbd, cache, w.B, ws)
    len_after, cur_after = cache.len, cache.cur
    for seed in (101, 102, 103, 104):
        q, k, v = data(seed)
        want = eager(q, k, v)                       # eager work (on the same workspace) between the replays
        sq.copy_(q); sk.copy_(k); sv.copy_(v)
        so.fill_(float("nan"))
        for buf in cache.kbuf + cache.vbuf:         # the graph starts from an empty cache: occupancy is host state,
            buf.zero_()                             # the buffers are cleared as a fresh cache's are
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert lb.lococo_scan_status(cfg, ws) == 0
        assert torch.equal(so, want[0]), seed
        assert torch.equal(cache.kbuf[cur_after], want[1]) and torch.equal(cache.vbuf[cur_after], want[2]), seed
        assert (len_after, cur_after) == want[3:]
