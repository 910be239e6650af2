"""GPU parity of the instantiation and the launch forms the benchmark line runs on: the 64-slot build
of the fused compression kernel under PEAKED softmax rows (near-uniform rows hide indexing mistakes),
the one-launch scan's fall-backs, step 3 alone on the MFMA kernels, and token selection through the
MFMA form of Eq. 6 + Eq. 4."""
import numpy as np
import pytest
import torch

from oracle import lococo_oracle as orc
from paper_2406_05317_amd import binding as lb
from paper_2406_05317_amd import inputs
from parity_util import TOL, assert_close, compare_scan, gpu_forward, oracle_forward, to_np

pytestmark = pytest.mark.gpu
MFMA = 2


def _w(**kw):
    base = dict(name="headline", dtype="bf16", batch=1, n_q_heads=4, n_kv_heads=4, head_dim=128, L=512,
                B=128, M=128, conv_width=15, seed=7)
    base.update(kw)
    return inputs.Workload(**base)


def _peak_of_first_compress(w, k, cw):
    """Largest normalised weight of the first compress step of chain (0, 0), by the oracle."""
    fills = w.M // w.B
    T = fills * w.B + w.B
    lg = orc.conv_logits(k[0, 0, :T].double().numpy(), (cw[0] if cw.dim() == 4 else cw).double().numpy())
    return orc.normalise(lg).max(), T


@pytest.mark.parametrize("gains", [(6.0, 3.0), (10.0, 8.0)])
@pytest.mark.parametrize("history", [True, False])
def test_64_slot_build_under_peaked_rows(gains, history):
    """64 chains x 4 tiles of 64 slots fill the compute units, so the build the headline number runs on
    is the one tested; sharpened Q, K and filters make both softmaxes peaked."""
    qk, cg = gains
    w = _w(batch=2, n_q_heads=32, n_kv_heads=32, M=256, B=128, L=640, qk_gain=qk, conv_gain=cg)
    cfg = lb.config_for(w, impl=MFMA)
    info = lb.lococo_describe_path(cfg, w.B)
    assert info["path"] == 1 and info["tile_slots"] == 64 and info["position_split"] == 1, info
    if history:
        assert info["scan_groups"] == w.batch * w.n_kv_heads, info      # one launch, one chain per workgroup
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    peak, T = _peak_of_first_compress(w, k, cw)
    assert peak > 20.0 / T, (peak, T)                     # far from the uniform 1 / T
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16)
    got = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=history)
    errs = compare_scan(w, got, want, what=f"64-slot build, gains {gains}")
    print(gains, history, "peak weight %.3f" % peak, {k_: (f"{e[0]:.2e}", f"{e[1]:.2e}") for k_, e in errs.items()})


def test_headline_shape_under_peaked_rows():
    """The benchmark shape itself (32 chains, M = B = 512: 256 workgroups of 64 slots, one launch for
    the scan), six blocks, sharpened."""
    w = _w(batch=1, n_q_heads=32, n_kv_heads=32, M=512, B=512, L=6 * 512, qk_gain=6.0, conv_gain=4.0)
    cfg = lb.config_for(w)
    info = lb.lococo_describe_path(cfg, w.B)
    assert info["path"] == 1 and info["tile_slots"] == 64 and info["scan_groups"] == 32, info
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    peak, T = _peak_of_first_compress(w, k, cw)
    assert peak > 20.0 / T, (peak, T)
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16)
    got = gpu_forward(w, q, k, v, cw, cb, history=True)
    errs = compare_scan(w, got, want, what="cfg3 shape, sharpened")
    print("peak weight %.3f" % peak, {k_: (f"{e[0]:.2e}", f"{e[1]:.2e}") for k_, e in errs.items()})


def _scan_with_launch_count(w, q, k, v, cw, cb, stream=None):
    lb.lococo_timing_begin()
    got = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True)
    ran = lb.lococo_timing_end()
    return got, ran["compress_mfma"][0]


def test_scan_falls_back_to_one_launch_per_step_when_the_grid_is_not_resident(options):
    """The one-launch scan needs its whole grid resident.  The occupancy figure is forced from the
    host to a value below the grid: every step then gets a launch of its own, and the results are
    the same bit for bit."""
    w = _w(M=256, B=128, L=1536, n_q_heads=8, n_kv_heads=8)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    cfg = lb.config_for(w, impl=MFMA)
    n_compress = sum(r[2] for r in lb.lococo_plan(w.L, w.B, w.M))
    info = lb.lococo_describe_path(cfg, w.B)
    assert info["scan_groups"] > 0 and info["scan_resident_limit"] >= info["compute_units"], info
    a, launches = _scan_with_launch_count(w, q, k, v, cw, cb)
    assert launches == 1
    options(lb.LOCOCO_OPT_MAX_RESIDENT, 8)
    assert lb.lococo_describe_path(cfg, w.B)["scan_groups"] == 0
    b, launches = _scan_with_launch_count(w, q, k, v, cw, cb)
    assert launches == n_compress
    for x, y in zip(a[:3], b[:3]):
        assert torch.equal(x, y)
    assert a[3:] == b[3:]


def test_a_second_scan_on_another_stream_does_not_start_a_second_persistent_launch():
    """Two scans in flight on two streams of one device: the second takes one launch per step, so two
    persistent grids never compete for the compute units.  Both results are right."""
    w = _w(M=256, B=128, L=1536, n_q_heads=8, n_kv_heads=8)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    n_compress = sum(r[2] for r in lb.lococo_plan(w.L, w.B, w.M))
    ref = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True)
    cfg = lb.config_for(w, impl=MFMA)
    dev = "cuda"
    qd, kd, vd, cwd, cbd = (t.to(dev) for t in (q, k, v, cw, cb))
    runs = []
    for _ in range(2):
        runs.append(dict(o=torch.full_like(qd, float("nan")), cache=lb.Cache(cfg, dev),
                         ws=lb.workspace(cfg, w.L, w.B, True, dev), stream=torch.cuda.Stream()))
    torch.cuda._sleep(1000)                               # (its first use loads the kernel and waits for it)
    torch.cuda.synchronize()
    lb.lococo_timing_begin()                              # (reading the timing waits for the device: once, at the end)
    for i, r in enumerate(runs):
        with torch.cuda.stream(r["stream"]):
            if i == 0:
                torch.cuda._sleep(200_000_000)            # the first scan sits behind ~80 ms of other work
            lb.lococo_sequence_forward(cfg, qd, kd, vd, r["o"], cwd, cbd, r["cache"], w.B, r["ws"])
    launches = lb.lococo_timing_end()["compress_mfma"][0]
    torch.cuda.synchronize()
    assert launches == 1 + n_compress, launches
    for r in runs:
        assert lb.lococo_scan_status(cfg, r["ws"]) == 0
        assert torch.equal(r["o"].cpu(), ref[0])
        assert torch.equal(r["cache"].k.cpu(), ref[1]) and torch.equal(r["cache"].v.cpu(), ref[2])


@pytest.mark.parametrize("m", [0, 17, 100, 128])
@pytest.mark.parametrize("B", [1, 96, 128])
def test_attn_only_on_the_mfma_kernels(m, B):
    """Step 3 alone at head_dim 128 / bf16: the tiled MFMA kernel (or, for one token, the
    generation-stage kernel), ragged cache occupancies, GQA."""
    w = _w(batch=2, n_q_heads=8, n_kv_heads=4, M=128, B=B, L=B)
    q, k, v = inputs.qkv(w)
    rng = np.random.default_rng(5)
    shape = (w.batch, w.n_kv_heads, w.M, w.head_dim)
    ck = torch.from_numpy(rng.standard_normal(shape) / np.sqrt(w.head_dim)).to(w.torch_dtype)
    cv = torch.from_numpy(rng.standard_normal(shape)).to(w.torch_dtype)
    cfg = lb.config_for(w)
    cache = lb.Cache(cfg)
    cache.load(ck.cuda(), cv.cuda(), m)
    k0, v0 = cache.k.clone(), cache.v.clone()
    o = torch.full(q.shape, float("nan"), dtype=w.torch_dtype, device="cuda")
    lb.lococo_timing_begin()
    lb.lococo_attn_only(cfg, q.cuda(), k.cuda(), v.cuda(), o, cache)
    ran = lb.lococo_timing_end()
    torch.cuda.synchronize()
    assert set(ran) == {"attn_decode" if B == 1 else "attn_mfma"}, ran
    assert cache.len == m and cache.cur == 0
    assert torch.equal(cache.k, k0) and torch.equal(cache.v, v0)      # never mutates the cache
    g = w.group
    for b in range(w.batch):
        for h in range(w.n_q_heads):
            want = orc.attention_block(q[b, h], k[b, h // g], v[b, h // g], ck[b, h // g, :m], cv[b, h // g, :m])
            assert_close(to_np(o[b, h]), want, TOL["bf16"], f"attn_only b{b} h{h} m{m} B{B}")


@pytest.mark.parametrize("shape", [dict(M=64, B=32), dict(M=128, B=64, batch=2, n_kv_heads=8), dict(M=256, B=256)])
def test_one_hot_logits_select_tokens_bit_exactly_on_the_mfma_kernel(shape):
    """Token dropping as a special case of the compression: one-hot rows through the MFMA form of
    Eq. 6 + Eq. 4 (weights 1 and 0 are exact in bf16) copy the selected entries bit for bit; slot i
    <- entry i + B keeps the last M tokens, block after block."""
    w = _w(n_q_heads=shape.get("n_kv_heads", 4), n_kv_heads=shape.get("n_kv_heads", 4), batch=shape.get("batch", 1),
           M=shape["M"], B=shape["B"], L=shape["M"] + 5 * shape["B"])
    _, k, v = inputs.qkv(w)
    cfg = lb.config_for(w)
    cache = lb.Cache(cfg)
    kd, vd = k.cuda(), v.cuda()
    cache.load(kd[:, :, :w.M].contiguous(), vd[:, :, :w.M].contiguous(), w.M)
    T = w.M + w.B
    logits = torch.full((w.batch, w.n_kv_heads, w.M, T), -1e30, dtype=torch.float32, device="cuda")
    logits[:, :, torch.arange(w.M), torch.arange(w.M) + w.B] = 0.0
    lb.lococo_timing_begin()
    for s in range(w.M, w.L, w.B):
        lb.lococo_mix_from_logits(cfg, kd[:, :, s:s + w.B], vd[:, :, s:s + w.B], logits, cache)
    ran = lb.lococo_timing_end()
    torch.cuda.synchronize()
    assert set(ran) == {"mix_mfma"}, ran
    assert cache.len == w.M and cache.cur == ((w.L - w.M) // w.B) % 2
    assert torch.equal(cache.k.cpu(), k[:, :, w.L - w.M:])           # bit-exact copies, in order
    assert torch.equal(cache.v.cpu(), v[:, :, w.L - w.M:])
    # and a scattered selection with -inf elsewhere: slot i <- entry perm[i]
    rng = np.random.default_rng(11)
    perm = torch.from_numpy(rng.permutation(T)[:w.M].copy()).cuda()
    logits = torch.full((w.batch, w.n_kv_heads, w.M, T), float("-inf"), dtype=torch.float32, device="cuda")
    logits[:, :, torch.arange(w.M), perm] = 3.5
    before_k, before_v = cache.k.clone(), cache.v.clone()
    blk_k, blk_v = kd[:, :, :w.B], vd[:, :, :w.B]
    lb.lococo_mix_from_logits(cfg, blk_k, blk_v, logits, cache)
    torch.cuda.synchronize()
    cat_k, cat_v = torch.cat([before_k, blk_k], 2), torch.cat([before_v, blk_v], 2)
    assert torch.equal(cache.k, cat_k[:, :, perm]) and torch.equal(cache.v, cat_v[:, :, perm])


@pytest.mark.parametrize("name,pipe,split", [("cfg2", 2, 1), ("cfg5", 2, 2), ("cfg3", 1, 1), ("cfg4", 1, 1)])
def test_which_shapes_use_idle_compute_units(name, pipe, split, options):
    """The 3.5 K-token workload and the GQA workload (128 (chain, slot tile) pairs each) leave half of the
    compute units without a pair: two workgroups per pair take the steps of the scan in turn.  Without that
    (a test hook), two workgroups share out the positions of every step of the GQA workload; the 3.5 K-token
    shape (M = 128: four position tiles of cache) is too short for that hand-over to pay."""
    w = inputs.CONFIGS[name]
    info = lb.lococo_describe_path(lb.config_for(w), w.B)
    assert info["step_pipeline"] == pipe and info["position_split"] == 1, info
    if info["compute_units"] == 256:
        assert info["scan_groups"] > 0, info
    options(lb.LOCOCO_OPT_NO_STEP_PIPELINE, 1)
    info = lb.lococo_describe_path(lb.config_for(w), w.B)
    assert info["step_pipeline"] == 1 and info["position_split"] == split, info


@pytest.mark.parametrize("case", [
    dict(M=256, B=256, L=1280, n_q_heads=8, n_kv_heads=4, batch=2),                      # cfg5-shaped, cut down: two parts
    dict(M=512, B=512, L=2048, n_q_heads=2, n_kv_heads=2),                               # four parts
    dict(M=256, B=200, L=1100, n_q_heads=4, n_kv_heads=4, qk_gain=6.0, conv_gain=4.0),   # peaked rows, ragged blocks, T = 456
    dict(M=256, B=96, L=800, n_q_heads=4, n_kv_heads=2),                                 # partly filled cache at the first compress
    dict(M=256, B=40, L=600, n_q_heads=4, n_kv_heads=2),                                 # short blocks: the last part nearly empty
    dict(M=256, B=128, L=896, norm=1, bias_sigma=0.5),                                   # relu-sum
    dict(M=256, B=128, L=896, conv_width=21, per_head_filters=True, bias_sigma=0.5),     # width 21, per-head banks
    dict(M=256, B=128, L=896, protect_share=0.15),                                       # protected slots
    dict(M=512, B=300, L=1500, norm=1, conv_width=21, protect_share=0.1, bias_sigma=0.3, n_q_heads=2, n_kv_heads=2),
])
def test_split_steps_match_the_oracle_and_every_schedule(case, options):
    """Shapes whose (chain, slot tile) pairs leave compute units idle share out the positions of a step
    between several workgroups, which leave partial results in the workspace for the last of them to
    merge.  Equal to the oracle; bit-identical between one launch per scan, one launch per step, block
    by block through lococo_segment_step, and either form of the hand-off."""
    case = dict(case)
    share = case.pop("protect_share", 0.0)
    w = _w(**case)
    cfg = lb.config_for(w, impl=MFMA)
    options(lb.LOCOCO_OPT_NO_STEP_PIPELINE, 1)       # (by default such shapes pair their workgroups over the steps instead)
    info = lb.lococo_describe_path(cfg, w.B)
    assert info["position_split"] > 1 and info["tile_slots"] == 32, info
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    protect = (np.random.default_rng(5).random((w.batch, w.n_kv_heads, w.M)) < share) if share else None
    a = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True, protect=protect)
    b = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=False, protect=protect)
    c = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, step_by_step=True, protect=protect)
    options(lb.LOCOCO_OPT_CHAIN_SYNC_DEVICE, 1)
    d = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True, protect=protect)
    e = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=False, protect=protect)
    options(lb.LOCOCO_OPT_CHAIN_SYNC_DEVICE, 0)
    options(lb.LOCOCO_OPT_SCAN_PER_STEP, 1)
    f = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=3, protect=protect)
    for other in (b, c, d, e, f):
        for x, y in zip(a[:3], other[:3]):
            assert torch.equal(x, y)
        assert a[3:] == other[3:]
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16, protect=protect)
    errs = compare_scan(w, a, want, what="split steps")
    print(case, info["position_split"], {k_: (f"{e_[0]:.2e}", f"{e_[1]:.2e}") for k_, e_ in errs.items()})


PIPE_CASES = [
    dict(M=128, B=128, L=1024),                                                          # the 3.5 K-token shape cut down: three block-only tiles, the chain met inside the prologue
    dict(M=256, B=256, L=2048, n_q_heads=8, n_kv_heads=4, batch=2),                      # the GQA shape cut down: seven block-only tiles, met before stage 3
    dict(M=128, B=160, L=1000),                                                          # four block-only tiles: met before stage 0; ragged last block
    dict(M=256, B=64, L=900, n_q_heads=4, n_kv_heads=2),                                 # short blocks: one block-only tile, met at once; four fills
    dict(M=128, B=96, L=700, qk_gain=6.0, conv_gain=4.0),                                # peaked rows; partly filled cache at the first compress
    dict(M=256, B=200, L=1100, norm=1, bias_sigma=0.5),                                  # relu-sum, T = 456
    dict(M=128, B=128, L=896, conv_width=21, per_head_filters=True, bias_sigma=0.5),     # width 21, per-head banks
    dict(M=256, B=128, L=896, protect_share=0.15),                                       # protected slots
    dict(M=128, B=128, L=896, conv_in=1, conv_width=21, norm=1, bias_sigma=0.4),         # [K | V] filters: two walks per turn
    dict(M=512, B=512, L=3072, n_q_heads=4, n_kv_heads=4),                               # 64 pairs, 32 position tiles
]


@pytest.mark.parametrize("case", PIPE_CASES, ids=[str(i) for i in range(len(PIPE_CASES))])
def test_pairs_of_workgroups_that_take_the_steps_in_turn(case, options):
    """Shapes with at most half as many (chain, slot tile) pairs as compute units: two workgroups per pair, each
    taking every other step of the scan and walking its step from the last position tile down, so that the
    block-only tiles are done while the partner finishes the step before.  Equal to the oracle; bit-identical
    between one launch per scan, one launch per step, block by block through lococo_segment_step (where one
    workgroup of each pair idles), windows of three blocks, and either form of the chain meeting.  The same
    shapes without the pairs (a test hook) meet the same tolerance."""
    case = dict(case)
    share = case.pop("protect_share", 0.0)
    w = _w(**case)
    cfg = lb.config_for(w, impl=MFMA)
    info = lb.lococo_describe_path(cfg, w.B)
    assert info["step_pipeline"] == 2 and info["position_split"] == 1 and info["tile_slots"] == 32, info
    if info["compute_units"] == 256:
        assert info["scan_groups"] > 0, info
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    protect = (np.random.default_rng(5).random((w.batch, w.n_kv_heads, w.M)) < share) if share else None
    a = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True, protect=protect)
    b = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=False, protect=protect)
    c = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, step_by_step=True, protect=protect)
    d = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=3, protect=protect)
    options(lb.LOCOCO_OPT_CHAIN_SYNC_DEVICE, 1)
    e = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True, protect=protect)
    options(lb.LOCOCO_OPT_CHAIN_SYNC_DEVICE, 0)
    options(lb.LOCOCO_OPT_SCAN_PER_STEP, 1)
    f = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True, protect=protect)
    options(lb.LOCOCO_OPT_SCAN_PER_STEP, 0)
    for other in (b, c, d, e, f):
        for x, y in zip(a[:3], other[:3]):
            assert torch.equal(x, y)
        assert a[3:] == other[3:]
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16, protect=protect)
    errs = compare_scan(w, a, want, what="steps in turn")
    print(case, {k_: (f"{e_[0]:.2e}", f"{e_[1]:.2e}") for k_, e_ in errs.items()})
    options(lb.LOCOCO_OPT_NO_STEP_PIPELINE, 1)
    assert lb.lococo_describe_path(cfg, w.B)["step_pipeline"] == 1
    g = gpu_forward(w, q, k, v, cw, cb, impl=MFMA, history=True, protect=protect)
    compare_scan(w, g, want, what="without the pairs")


def test_split_generation_steps(options):
    """B = 1 on a shape that splits: T = M + 1, the last part holds the new token's tile."""
    w = _w(M=512, B=128, L=512 + 10, n_q_heads=4, n_kv_heads=2)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    cfg = lb.config_for(w, impl=MFMA)
    options(lb.LOCOCO_OPT_NO_STEP_PIPELINE, 1)
    assert lb.lococo_describe_path(cfg, 1)["position_split"] > 1
    sl = lambda t, a_, b_: t[:, :, a_:b_]
    P = 512
    o1, ck, cv, ln = oracle_forward(w, sl(q, 0, P), sl(k, 0, P), sl(v, 0, P), cw, cb, nthreads=16)
    o2, ck, cv, ln = oracle_forward(w, sl(q, P, w.L), sl(k, P, w.L), sl(v, P, w.L), cw, cb, B=1, cache=(ck, cv, ln), nthreads=16)
    want = (np.concatenate([o1, o2], 2), ck, cv, ln)
    qd, kd, vd, cwd, cbd = (t.cuda() for t in (q, k, v, cw, cb))
    od = torch.full_like(qd, float("nan"))
    cache = lb.Cache(cfg)
    lb.lococo_sequence_forward(cfg, sl(qd, 0, P), sl(kd, 0, P), sl(vd, 0, P), sl(od, 0, P), cwd, cbd, cache, w.B,
                               lb.workspace(cfg, P, w.B, True))
    ws1 = lb.workspace(cfg, 1, 1, False)
    for t in range(P, w.L):
        lb.lococo_segment_step(cfg, sl(qd, t, t + 1), sl(kd, t, t + 1), sl(vd, t, t + 1), sl(od, t, t + 1), cwd, cbd, cache, ws1)
    torch.cuda.synchronize()
    compare_scan(w, (od.cpu(), cache.k.cpu(), cache.v.cpu(), cache.len, cache.cur), want, what="split decode")
