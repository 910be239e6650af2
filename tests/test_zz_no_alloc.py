"""lococo_segment_step_noalloc (the step on the library's own scratch array, for callers that cannot
allocate) against lococo_segment_step with a caller-owned workspace: same kernels, so the same bits,
on two calls in a row, the second with a smaller input (the array keeps what the first call left)."""
import numpy as np
import pytest
import torch

from paper_2406_05317_amd import binding as lb
from paper_2406_05317_amd import inputs

pytestmark = pytest.mark.gpu


def _w(**kw):
    base = dict(name="noalloc", dtype="bf16", batch=2, n_q_heads=8, n_kv_heads=4, head_dim=128, L=256,
                B=128, M=128, conv_width=15, seed=21)
    base.update(kw)
    return inputs.Workload(**base)


def _one_step(w, B, noalloc, track=False):
    """One compress step of B tokens from a full, seeded cache.  Returns (o, cache_k, cache_v, len, cur, colsum)."""
    cfg = lb.config_for(w)
    q, k, v = inputs.qkv(w, B)
    cw, cb = inputs.conv_filters(w)
    qd, kd, vd, cwd, cbd = (t.cuda() for t in (q, k, v, cw, cb))
    rng = np.random.default_rng(3)
    shape = (w.batch, w.n_kv_heads, w.M, w.head_dim)
    cache = lb.Cache(cfg)
    cache.load(torch.from_numpy(rng.standard_normal(shape) / 11.0).to(w.torch_dtype).cuda(),
               torch.from_numpy(rng.standard_normal(shape)).to(w.torch_dtype).cuda(), w.M)
    if track:
        cache.track_attention()
    od = torch.full_like(qd, float("nan"))
    if noalloc:
        lb.lococo_segment_step_noalloc(cfg, qd, kd, vd, od, cwd, cbd, cache)
    else:
        lb.lococo_segment_step(cfg, qd, kd, vd, od, cwd, cbd, cache, lb.workspace(cfg, B, B, False))
    torch.cuda.synchronize()
    return (od.cpu(), cache.k.cpu(), cache.v.cpu(), cache.len, cache.cur,
            None if cache.attn_colsum is None else cache.attn_colsum.cpu())


@pytest.mark.parametrize("case", [
    dict(),                                                  # fused MFMA kernel: repacked filters in the array
    dict(conv_width=7),                                      # unfused MFMA path: packed filters, statistics, logits
    dict(dtype="f32", head_dim=32, M=40, conv_width=5),      # shape-agnostic kernels: the logits
])
def test_noalloc_step_equals_the_step_with_a_workspace_twice_in_a_row(case):
    w = _w(**case)
    B1 = 128 if w.head_dim == 128 else 24
    second = w.replace(batch=1, n_q_heads=4, n_kv_heads=2, seed=22)      # fewer chains, fewer tokens
    B2 = 64 if w.head_dim == 128 else 9
    for (wl, B, track) in ((w, B1, False), (second, B2, True)):
        want = _one_step(wl, B, noalloc=False, track=track)
        got = _one_step(wl, B, noalloc=True, track=track)
        assert torch.isfinite(got[0].float()).all()
        for x, y in zip(got[:3], want[:3]):
            assert torch.equal(x, y)
        assert got[3:5] == want[3:5] == (wl.M, 1)
        if track:       # summed with floating-point atomics: equal up to the order of the additions
            assert torch.allclose(got[5], want[5], rtol=1e-5, atol=0.0) and float(want[5].min()) > 0.0


def test_noalloc_step_refuses_what_does_not_fit_or_cannot_be_shared():
    import ctypes as C
    big = _w(dtype="f32", batch=4, n_q_heads=32, n_kv_heads=32, head_dim=64, M=256, conv_width=5)   # 128 MB of logits
    cfg = lb.config_for(big)
    assert lb.lococo_workspace_bytes(cfg, 256, 256) > (16 << 20)
    q, k, v = (torch.zeros((4, 32, 256, 64), device="cuda") for _ in range(3))
    o = torch.zeros_like(q)
    cw = torch.zeros((256, 64, 5), device="cuda")
    cache = lb.Cache(cfg)
    cache.c.len = 256
    with pytest.raises(lb.LococoError) as e:
        lb.lococo_segment_step_noalloc(cfg, q, k, v, o, cw, None, cache)
    assert e.value.status == lb.LOCOCO_EWORKSPACE and cache.len == 256 and cache.cur == 0
    w = _w()
    cfg = lb.config_for(w, flags=lb.LOCOCO_FLAG_FILTERS_PREPARED)
    cache = lb.Cache(cfg)
    with pytest.raises(lb.LococoError) as e:
        lb.lococo_segment_step_noalloc(cfg, *(torch.zeros((2, 8, 128, 128), dtype=torch.bfloat16, device="cuda"),
                                               torch.zeros((2, 4, 128, 128), dtype=torch.bfloat16, device="cuda"),
                                               torch.zeros((2, 4, 128, 128), dtype=torch.bfloat16, device="cuda"),
                                               torch.zeros((2, 8, 128, 128), dtype=torch.bfloat16, device="cuda")),
                                       torch.zeros((128, 128, 15), dtype=torch.bfloat16, device="cuda"), None, cache)
    assert e.value.status == lb.LOCOCO_EINVAL
