"""GPU parity of protected cache slots (the combination with an eviction policy: attention sinks,
heavy hitters) against the CPU oracle, on the shape-agnostic kernels and on the MFMA kernels."""
import numpy as np
import pytest
import torch

from oracle import lococo_oracle as orc
from paper_2406_05317_amd import inputs
from parity_util import compare_scan, gpu_forward, oracle_forward

pytestmark = pytest.mark.gpu


def _masks(w, kind, seed=5):
    rng = np.random.default_rng(seed)
    if kind == "sinks":                                   # the first four tokens, every chain
        m = np.zeros(w.M, bool)
        m[:4] = True
    elif kind == "first_tile":                            # a whole 32-position tile protected
        m = np.zeros(w.M, bool)
        m[:32] = True
    elif kind == "scattered":                             # heavy-hitter-like: different slots per chain
        m = rng.random((w.batch, w.n_kv_heads, w.M)) < 0.15
    elif kind == "all":
        m = np.ones(w.M, bool)
    else:
        raise ValueError(kind)
    return m


def _run(w, kind, **kw):
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    prot = _masks(w, kind)
    want = oracle_forward(w, q, k, v, cw, cb, nthreads=16, protect=prot)
    got = gpu_forward(w, q, k, v, cw, cb, protect=prot, **kw)
    errs = compare_scan(w, got, want, what=f"protect/{kind}")
    # a protected slot that was filled by a token (live before the first compression) still holds
    # that token: bit-identical on both sides, whatever the tolerance
    plan = orc.plan(w.L, w.B, w.M)
    m_first = int(plan[plan[:, 2] == 1][0, 3]) if (plan[:, 2] == 1).any() else w.M
    full = np.broadcast_to(prot, (w.batch, w.n_kv_heads, w.M)).copy()
    full[..., m_first:] = False
    ck, cv = got[1].double().numpy(), got[2].double().numpy()
    assert full.any()
    assert np.array_equal(ck[full], want[1][full]) and np.array_equal(cv[full], want[2][full])
    tok = np.nonzero(full)
    assert np.array_equal(ck[full], k.double().numpy()[tok[0], tok[1], tok[2]])
    # and the mask matters: without it the result differs
    if kind != "all":
        base = oracle_forward(w, q, k, v, cw, cb, nthreads=16)
        assert np.abs(base[1] - want[1]).max() > 1e-3
    return errs


@pytest.mark.parametrize("kind", ["sinks", "scattered", "all"])
@pytest.mark.parametrize("case", [
    dict(dtype="f32", batch=2, n_q_heads=4, n_kv_heads=2, head_dim=32, L=96, B=16, M=40, conv_width=5),
    dict(dtype="bf16", batch=1, n_q_heads=2, n_kv_heads=2, head_dim=64, L=160, B=32, M=64, conv_width=7, norm=1,
         bias_sigma=0.5),
    dict(dtype="f32", batch=1, n_q_heads=2, n_kv_heads=1, head_dim=16, L=70, B=12, M=20, conv_width=3, conv_in=1),
])
def test_generic_kernels_with_protected_slots(case, kind):
    w = inputs.Workload(name="protect", seed=3, **case)
    _run(w, kind, impl=1)


@pytest.mark.parametrize("kind", ["sinks", "first_tile", "scattered", "all"])
@pytest.mark.parametrize("case", [
    dict(),                                               # 32-slot tiles
    dict(L=500, B=96),                                    # partly filled cache at the first compress, ragged tail
    dict(batch=2, n_q_heads=32, n_kv_heads=32, M=256, L=512),        # 64-slot tiles
    dict(conv_width=21, norm=1, bias_sigma=0.5, M=96, B=80, L=400),
])
def test_mfma_kernels_with_protected_slots(case, kind):
    base = dict(name="protect", dtype="bf16", batch=1, n_q_heads=4, n_kv_heads=4, head_dim=128, L=512, B=128,
                M=128, conv_width=15, seed=7)
    base.update(case)
    w = inputs.Workload(**base)
    for history in (False, True):
        errs = _run(w, kind, impl=2, history=history)
    print(case, kind, {k: (f"{e[0]:.2e}", f"{e[1]:.2e}") for k, e in errs.items()})
