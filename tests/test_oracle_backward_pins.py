"""Pins of the oracle's backward pass: central finite differences of the oracle's FORWARD pass
(a different routine), for every input of one block step, in every branch and variant."""
import numpy as np
import pytest

from oracle import lococo_oracle as orc


def rand(rng, *shape, scale=1.0):
    return rng.standard_normal(shape) * scale


def _forward(q, kb, vb, ck, cv, m, cw, cb, M, **kw):
    """One block step through the forward oracle: (o, new_k, new_v)."""
    o, nk, nv, ln = orc.sequence_forward(q, kb, vb, cw, cb, B=q.shape[2], M=M, cache_k=ck, cache_v=cv,
                                         cache_len=m, **kw)
    return o, nk, nv, ln


CASES = {
    "compress_softmax": dict(b=1, Hq=2, Hkv=1, Bn=5, M=6, m=6, d=4, k=3),
    "compress_partial_cache": dict(b=1, Hq=1, Hkv=1, Bn=5, M=6, m=3, d=4, k=5),
    "compress_relu_sum": dict(b=1, Hq=1, Hkv=1, Bn=4, M=5, m=5, d=3, k=3, norm=1),
    "compress_kv_channels": dict(b=1, Hq=1, Hkv=1, Bn=4, M=5, m=5, d=3, k=3, conv_in=1),
    "compress_protected": dict(b=1, Hq=2, Hkv=2, Bn=4, M=6, m=6, d=3, k=3, protect=[1, 0, 0, 1, 0, 0]),
    "compress_per_head_filters": dict(b=2, Hq=2, Hkv=2, Bn=3, M=4, m=4, d=3, k=3, per_head=True),
    "fill": dict(b=1, Hq=2, Hkv=1, Bn=3, M=8, m=2, d=4, k=3),
}


@pytest.mark.parametrize("name", sorted(CASES))
def test_step_backward_matches_finite_differences_of_the_forward(name):
    c = dict(CASES[name])
    rng = np.random.default_rng(sum(name.encode()))
    b, Hq, Hkv, Bn, M, m, d, k = (c[x] for x in ("b", "Hq", "Hkv", "Bn", "M", "m", "d", "k"))
    norm, conv_in, protect = c.get("norm", 0), c.get("conv_in", 0), c.get("protect")
    C = d * (2 if conv_in else 1)
    q, kb, vb = rand(rng, b, Hq, Bn, d), rand(rng, b, Hkv, Bn, d), rand(rng, b, Hkv, Bn, d)
    ck, cv = rand(rng, b, Hkv, M, d), rand(rng, b, Hkv, M, d)
    ck[:, :, m:], cv[:, :, m:] = 0.0, 0.0
    cw = rand(rng, *((Hkv,) if c.get("per_head") else ()), M, C, k, scale=0.7)
    cb = rand(rng, *((Hkv,) if c.get("per_head") else ()), M, scale=0.5)
    r_o, r_k, r_v = rand(rng, b, Hq, Bn, d), rand(rng, b, Hkv, M, d), rand(rng, b, Hkv, M, d)
    kw = dict(norm=norm, conv_in=conv_in, protect=None if protect is None else np.array(protect, bool))

    def loss(q=q, kb=kb, vb=vb, ck=ck, cv=cv, cw=cw, cb=cb):
        o, nk, nv, ln = _forward(q, kb, vb, ck, cv, m, cw, cb, M, **kw)
        return (o * r_o).sum() + (nk[:, :, :ln] * r_k[:, :, :ln]).sum() + (nv[:, :, :ln] * r_v[:, :, :ln]).sum()

    ln = min(M, m + Bn) if m + Bn <= M else M
    gk, gv = r_k.copy(), r_v.copy()
    gk[:, :, ln:], gv[:, :, ln:] = 0.0, 0.0
    g = orc.step_backward(q, kb, vb, ck, cv, m, cw, cb, r_o, gk, gv, M=M, norm=norm, conv_in=conv_in,
                          protect=kw["protect"])
    names = dict(q="dq", kb="dk", vb="dv", ck="d_cache_k", cv="d_cache_v", cw="d_conv_w", cb="d_conv_b")
    arrays = dict(q=q, kb=kb, vb=vb, ck=ck, cv=cv, cw=cw, cb=cb)
    eps = 1e-6
    for key, arr in arrays.items():
        got = g[names[key]]
        live = np.ones(arr.shape, bool)
        if key in ("ck", "cv"):
            live[:, :, m:] = False                        # slots that are not live are no inputs
        idx = np.argwhere(live)
        pick = idx if len(idx) <= 60 else idx[rng.choice(len(idx), 60, replace=False)]
        for at in map(tuple, pick):
            hi, lo = arr.copy(), arr.copy()
            hi[at] += eps
            lo[at] -= eps
            fd = (loss(**{key: hi}) - loss(**{key: lo})) / (2 * eps)
            if m + Bn <= M and key in ("cw", "cb"):
                assert got[at] == 0.0                     # a fill step does not touch the filters
            else:
                assert abs(got[at] - fd) <= 2e-6 * max(1.0, abs(fd)), (name, key, at, got[at], fd)
        if key in ("ck", "cv"):
            assert not got[:, :, m:].any()


def test_filter_gradients_add_over_chains_and_calls():
    """d_conv_w of a shared bank is the sum over chains of the per-chain gradients."""
    rng = np.random.default_rng(5)
    b, H, Bn, M, d, k = 2, 2, 3, 4, 3, 3
    q, kb, vb = rand(rng, b, H, Bn, d), rand(rng, b, H, Bn, d), rand(rng, b, H, Bn, d)
    ck, cv, cw = rand(rng, b, H, M, d), rand(rng, b, H, M, d), rand(rng, M, d, k)
    do, gk, gv = rand(rng, b, H, Bn, d), rand(rng, b, H, M, d), rand(rng, b, H, M, d)
    whole = orc.step_backward(q, kb, vb, ck, cv, M, cw, None, do, gk, gv, M=M)
    parts = 0.0
    for bi in range(b):
        for h in range(H):
            s = (slice(bi, bi + 1), slice(h, h + 1))
            one = orc.step_backward(q[s], kb[s], vb[s], ck[s], cv[s], M, cw, None, do[s], gk[s], gv[s], M=M)
            parts = parts + one["d_conv_w"]
            np.testing.assert_allclose(one["dq"], whole["dq"][s], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(whole["d_conv_w"], parts, rtol=1e-12, atol=1e-13)
