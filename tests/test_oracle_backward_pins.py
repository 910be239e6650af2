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


def test_the_reverse_walk_over_a_scan_against_finite_differences_of_the_scan():
    """The composition the GPU scan backward is compared with (the step backward walked over the blocks in
    reverse, each block's gradient w.r.t. its starting state handed to the block before) against central
    differences of the forward oracle over the WHOLE scan: fills, compressions, a ragged last block, a
    cache that starts half full, protected slots."""
    from parity_util import oracle_scan_backward
    from paper_2406_05317_amd import inputs
    for seed, kw, len0, use_protect in (
            (1, dict(batch=2, n_q_heads=4, n_kv_heads=2, head_dim=8, L=41, B=8, M=14, conv_width=3), 0, False),
            (2, dict(batch=1, n_q_heads=2, n_kv_heads=2, head_dim=4, L=30, B=6, M=10, conv_width=3, norm=1,
                     bias_sigma=0.4, per_head_filters=True), 7, False),
            (3, dict(batch=1, n_q_heads=2, n_kv_heads=1, head_dim=6, L=24, B=8, M=8, conv_width=5, conv_in=1), 8, True)):
        w = inputs.Workload(name="walk", dtype="f32", seed=seed, conv_gain=3.0, **kw)
        rng = np.random.default_rng(seed)
        q, k, v = (t.double().numpy() for t in inputs.qkv(w))
        cw, cb = (t.double().numpy() for t in inputs.conv_filters(w))
        chains = (w.batch, w.n_kv_heads, w.M, w.head_dim)
        ck0, cv0 = rand(rng, *chains, scale=0.5), rand(rng, *chains, scale=0.5)
        ck0[:, :, len0:], cv0[:, :, len0:] = 0, 0
        r_o, r_k, r_v = rand(rng, *q.shape), rand(rng, *chains), rand(rng, *chains)
        protect = (rng.random(chains[:3]) < 0.3) if use_protect else None
        got = oracle_scan_backward(w, q, k, v, cw, cb, ck0, cv0, len0, r_o, r_k, r_v, protect)

        def loss(q_, k_, v_, cw_, cb_, ck_, cv_):
            o, ck, cv, _ = orc.sequence_forward(q_, k_, v_, cw_, cb_, B=w.B, M=w.M, conv_in=w.conv_in, norm=w.norm,
                                                cache_k=ck_, cache_v=cv_, cache_len=len0, protect=protect)
            return (o * r_o).sum() + (ck * r_k).sum() + (cv * r_v).sum()

        args = [q, k, v, cw, cb, ck0, cv0]
        names = ["dq", "dk", "dv", "d_conv_w", "d_conv_b", "d_cache0_k", "d_cache0_v"]
        eps = 1e-6
        for i, name in enumerate(names):
            direction = rand(rng, *args[i].shape)
            if name.startswith("d_cache0"):
                direction[:, :, len0:] = 0              # rows that are not live are not inputs
            hi = [a + eps * direction if j == i else a for j, a in enumerate(args)]
            lo = [a - eps * direction if j == i else a for j, a in enumerate(args)]
            fd = (loss(*hi) - loss(*lo)) / (2 * eps)
            mine = float((got[name] * direction).sum())
            assert abs(mine - fd) < 1e-6 * max(1.0, abs(fd)), (seed, name, mine, fd)
