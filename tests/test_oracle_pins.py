"""Pins for the CPU oracle: each test checks it against something the paper or
the mathematics fixes, coded here independently (numpy / torch library calls,
closed forms, brute force), never against the oracle itself.

Paper anchors: Eq. 1 (attention), Alg. 1 / Alg. 2 (segment scan and the IF
that fills the cache), Eq. 3-4 (fusion, shared weights), Eq. 5 (convolution),
Eq. 6 (normalisation), the "connection with token dropping" paragraph
(one-hot weights = selection) and the convolutional-heads paragraph of the
experimental settings (parameter count).
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import lococo_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------- helpers
def full_causal_attention(q, k, v):
    """Eq. 1 written with whole matrices: softmax over keys s <= t."""
    L, d = q.shape
    s = (q @ k.T) / math.sqrt(d)
    s = np.where(np.tril(np.ones((L, L), dtype=bool)), s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    p /= p.sum(axis=1, keepdims=True)
    return p @ v


def windowed_attention(q, k, v, B, M):
    """Query t of segment n sees the M tokens before its segment start plus the
    block tokens up to itself (what a cache holding the last M tokens gives)."""
    L, d = q.shape
    out = np.zeros_like(q)
    for t in range(L):
        seg0 = (t // B) * B
        lo = max(0, seg0 - M)
        ks, vs = k[lo:t + 1], v[lo:t + 1]
        s = ks @ q[t] / math.sqrt(d)
        p = np.exp(s - s.max())
        p /= p.sum()
        out[t] = p @ vs
    return out


def rand(rng, *shape, scale=1.0):
    return rng.standard_normal(shape) * scale


# ----------------------------------------------------------------- plan
def simulate_plan(L, B, M, len0, cur0):
    """Token-by-token replay of Alg. 2's loop and IF, written without any
    segment arithmetic: walk tokens, cut a block every B tokens."""
    rows, m, cur, block, start = [], len0, cur0, 0, 0
    for t in range(L):
        block += 1
        if block == B or t == L - 1:
            if m + block <= M:
                rows.append((start, block, 0, m, m + block, cur))
                m += block
            else:
                cur = 1 - cur
                rows.append((start, block, 1, m, M, cur))
                m = M
            start, block = t + 1, 0
    return np.array(rows, dtype=np.int64).reshape(-1, 6)


def test_plan_matches_simulation():
    rng = np.random.default_rng(0)
    cases = [(256, 16, 16, 0, 0), (3584, 128, 128, 0, 0), (32768, 512, 512, 0, 0),
             (8192, 64, 128, 0, 0), (16384, 256, 256, 0, 1), (0, 4, 4, 0, 0), (1, 4, 4, 4, 0),
             (7, 1, 3, 0, 0), (10, 16, 4, 0, 0), (100, 7, 24, 5, 1)]
    for _ in range(200):
        M = int(rng.integers(1, 40))
        cases.append((int(rng.integers(0, 300)), int(rng.integers(1, 50)), M,
                      int(rng.integers(0, M + 1)), int(rng.integers(0, 2))))
    for L, B, M, len0, cur0 in cases:
        got = orc.plan(L, B, M, len0, cur0)
        want = simulate_plan(L, B, M, len0, cur0)
        assert got.shape == want.shape, (L, B, M, len0)
        assert np.array_equal(got, want), (L, B, M, len0, cur0)


def test_plan_counts_of_the_measured_configs():
    # 1 fill + 15 compress, 1 + 27, 1 + 63, 2 + 126, 1 + 63
    for (L, B, M), (fills, comps) in {(256, 16, 16): (1, 15), (3584, 128, 128): (1, 27),
                                      (32768, 512, 512): (1, 63), (8192, 64, 128): (2, 126),
                                      (16384, 256, 256): (1, 63)}.items():
        p = orc.plan(L, B, M)
        assert (p[:, 2] == 0).sum() == fills and (p[:, 2] == 1).sum() == comps


# ----------------------------------------------------------------- attention
def test_attention_block_vs_sdpa_library():
    """Step 3 against torch's scaled_dot_product_attention with an explicit mask."""
    rng = np.random.default_rng(1)
    for m, Bn, d in [(0, 5, 8), (7, 5, 8), (16, 16, 64), (3, 1, 4)]:
        q, kb, vb = rand(rng, Bn, d), rand(rng, Bn, d), rand(rng, Bn, d)
        ck, cv = rand(rng, m, d), rand(rng, m, d)
        got = orc.attention_block(q, kb, vb, ck, cv)
        K = torch.from_numpy(np.concatenate([ck, kb]))
        V = torch.from_numpy(np.concatenate([cv, vb]))
        mask = torch.ones(Bn, m + Bn, dtype=torch.bool)
        mask[:, m:] = torch.tril(torch.ones(Bn, Bn, dtype=torch.bool))
        want = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(q)[None], K[None], V[None], attn_mask=mask[None])[0].numpy()
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_attention_special_cases():
    rng = np.random.default_rng(2)
    d = 8
    # one visible key -> its value, exactly
    q, kb, vb = rand(rng, 1, d), rand(rng, 1, d), rand(rng, 1, d)
    assert np.array_equal(orc.attention_block(q, kb, vb, np.zeros((0, d)), np.zeros((0, d))), vb)
    # all values equal -> output equals that value
    m, Bn = 6, 4
    vrow = rand(rng, 1, d)
    o = orc.attention_block(rand(rng, Bn, d), rand(rng, Bn, d), np.repeat(vrow, Bn, 0),
                            rand(rng, m, d), np.repeat(vrow, m, 0))
    np.testing.assert_allclose(o, np.repeat(vrow, Bn, 0), rtol=1e-13)
    # B = 1 with a full cache: textbook single-query softmax attention
    q, kb, vb = rand(rng, 1, d), rand(rng, 1, d), rand(rng, 1, d)
    ck, cv = rand(rng, m, d), rand(rng, m, d)
    K, V = np.concatenate([ck, kb]), np.concatenate([cv, vb])
    s = K @ q[0] / math.sqrt(d)
    p = np.exp(s - s.max()); p /= p.sum()
    np.testing.assert_allclose(orc.attention_block(q, kb, vb, ck, cv)[0], p @ V, rtol=1e-13)
    # the scale argument is used as given
    o2 = orc.attention_block(q, kb, vb, ck, cv, scale=0.0)
    np.testing.assert_allclose(o2[0], V.mean(0), rtol=1e-13)


def test_future_block_keys_are_invisible():
    rng = np.random.default_rng(3)
    m, Bn, d = 3, 6, 4
    q, kb, vb, ck, cv = (rand(rng, *s) for s in [(Bn, d)] * 3 + [(m, d)] * 2)
    base = orc.attention_block(q, kb, vb, ck, cv)
    kb2, vb2 = kb.copy(), vb.copy()
    kb2[4:] += 100.0
    vb2[4:] -= 50.0
    pert = orc.attention_block(q, kb2, vb2, ck, cv)
    assert np.array_equal(base[:4], pert[:4])         # rows 0..3 never see keys 4, 5
    assert not np.allclose(base[4:], pert[4:])


# ----------------------------------------------------------------- P1: scan that fits
@pytest.mark.parametrize("L,B,M", [(48, 16, 64), (50, 16, 64), (37, 5, 40), (16, 16, 16)])
def test_scan_equals_full_causal_attention_when_everything_fits(L, B, M):
    rng = np.random.default_rng(4)
    d, Hq, Hkv, b = 8, 4, 2, 2
    q, k, v = rand(rng, b, Hq, L, d), rand(rng, b, Hkv, L, d), rand(rng, b, Hkv, L, d)
    o, ck, cv, ln = orc.sequence_forward(q, k, v, None, B=B, M=M)
    assert ln == L
    for bi in range(b):
        for h in range(Hq):
            want = full_causal_attention(q[bi, h], k[bi, h // 2], v[bi, h // 2])
            np.testing.assert_allclose(o[bi, h], want, rtol=1e-11, atol=1e-13)
    # the fill branch keeps every pair, in order
    assert np.array_equal(ck[:, :, :L], k) and np.array_equal(cv[:, :, :L], v)


def test_prefix_before_first_compression_is_full_attention():
    """The first compression only changes what later segments see."""
    rng = np.random.default_rng(5)
    L, B, M, d = 96, 8, 24, 8
    q, k, v = rand(rng, 1, 1, L, d), rand(rng, 1, 1, L, d), rand(rng, 1, 1, L, d)
    cw = rand(rng, M, d, 3)
    o, *_ = orc.sequence_forward(q, k, v, cw, B=B, M=M)
    n_exact = (M // B + 1) * B
    want = full_causal_attention(q[0, 0], k[0, 0], v[0, 0])
    np.testing.assert_allclose(o[0, 0, :n_exact], want[:n_exact], rtol=1e-11, atol=1e-13)
    assert not np.allclose(o[0, 0, n_exact:], want[n_exact:], rtol=1e-3)


# ----------------------------------------------------------------- conv (Eq. 5)
@pytest.mark.parametrize("T,C,M,k", [(20, 6, 5, 3), (9, 4, 7, 15), (33, 8, 4, 1), (5, 3, 2, 21)])
def test_conv_logits_vs_library_conv1d(T, C, M, k):
    rng = np.random.default_rng(6)
    X, Wc, bias = rand(rng, T, C), rand(rng, M, C, k), rand(rng, M)
    got = orc.conv_logits(X, Wc, bias)
    want = torch.nn.functional.conv1d(torch.from_numpy(X.T.copy())[None], torch.from_numpy(Wc),
                                      torch.from_numpy(bias), padding=(k - 1) // 2)[0].numpy()
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_conv_width_one_is_a_matrix_product_and_no_bias_is_zero_bias():
    rng = np.random.default_rng(7)
    X, Wc = rand(rng, 11, 5), rand(rng, 4, 5, 1)
    np.testing.assert_allclose(orc.conv_logits(X, Wc), Wc[:, :, 0] @ X.T, rtol=1e-13, atol=1e-14)


def test_conv_definition_by_hand_on_a_tiny_case():
    # M=1, C=1, k=3, taps (1, 10, 100): W[j] = x[j-1] + 10 x[j] + 100 x[j+1], zeros outside
    X = np.array([[1.0], [2.0], [3.0], [4.0]])
    Wc = np.array([[[1.0, 10.0, 100.0]]])
    got = orc.conv_logits(X, Wc)
    assert np.array_equal(got, np.array([[210.0, 321.0, 432.0, 43.0]]))


def test_conv_linearity_and_interior_shift_equivariance():
    rng = np.random.default_rng(8)
    T, C, M, k = 40, 3, 4, 7
    X1, X2, Wc = rand(rng, T, C), rand(rng, T, C), rand(rng, M, C, k)
    a, b = 0.7, -1.3
    np.testing.assert_allclose(orc.conv_logits(a * X1 + b * X2, Wc),
                               a * orc.conv_logits(X1, Wc) + b * orc.conv_logits(X2, Wc),
                               rtol=1e-11, atol=1e-12)
    s = 5
    Xs = np.zeros_like(X1)
    Xs[s:] = X1[:-s]
    W0, Ws = orc.conv_logits(X1, Wc), orc.conv_logits(Xs, Wc)
    pad = (k - 1) // 2
    np.testing.assert_allclose(Ws[:, s + pad:T - pad], W0[:, pad:T - pad - s], rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------- normalisation (Eq. 6)
def test_normalised_rows_sum_to_one_and_match_library_softmax():
    rng = np.random.default_rng(9)
    W = rand(rng, 6, 37, scale=4.0)
    w = orc.normalise(W, norm=0)
    assert np.all(w > 0) and np.all(w <= 1)
    np.testing.assert_allclose(w.sum(1), 1.0, rtol=0, atol=1e-14)
    np.testing.assert_allclose(w, torch.softmax(torch.from_numpy(W), dim=1).numpy(), rtol=1e-13)
    # literal Eq. 6 with a ReLU in front: relu(W) / (sum relu(W) + eps)
    eps = 1e-6
    w1 = orc.normalise(W, norm=1, eps=eps)
    r = np.maximum(W, 0)
    np.testing.assert_allclose(w1, r / (r.sum(1, keepdims=True) + eps), rtol=1e-13)
    assert np.all(w1 >= 0) and np.all(np.abs(w1.sum(1) - 1) < 1e-5)


def test_softmax_is_stable_for_huge_logits():
    W = np.array([[1e4, 1e4 - 1.0, -1e4]])
    w = orc.normalise(W)
    np.testing.assert_allclose(w[0, :2], [1 / (1 + math.exp(-1)), math.exp(-1) / (1 + math.exp(-1))],
                               rtol=1e-13)
    assert w[0, 2] == 0.0


# ----------------------------------------------------------------- mix (Eq. 4)
def test_mix_is_a_matrix_product():
    rng = np.random.default_rng(10)
    w, Y = rand(rng, 5, 9), rand(rng, 9, 4)
    np.testing.assert_allclose(orc.mix(w, Y), w @ Y, rtol=1e-13, atol=1e-14)


# ----------------------------------------------------------------- scan-level pins
def _one_hot_logits(n_steps, b, Hkv, M, B, sel):
    """sel(i, T) -> selected position for slot i when T entries are present."""
    lo = np.full((n_steps, b, Hkv, M, M + B), -np.inf)
    for i in range(M):
        lo[:, :, :, i, sel(i)] = 0.0
    return lo


def test_one_hot_weights_select_tokens_and_give_sliding_window_attention():
    """Token dropping as a special case of the compression operator: slot i takes
    entry i + B of [cache; block], so the cache is always the last M tokens."""
    rng = np.random.default_rng(11)
    L, B, M, d, b, Hq, Hkv = 80, 8, 16, 4, 1, 2, 1
    q, k, v = rand(rng, b, Hq, L, d), rand(rng, b, Hkv, L, d), rand(rng, b, Hkv, L, d)
    p = orc.plan(L, B, M)
    n_steps = int((p[:, 2] == 1).sum())
    lo = _one_hot_logits(n_steps, b, Hkv, M, B, lambda i: i + B)
    o, ck, cv, ln = orc.sequence_forward(q, k, v, None, B=B, M=M, logits_override=lo)
    assert ln == M
    assert np.array_equal(ck[0, 0], k[0, 0, L - M:])      # bit-exact copies, in order
    assert np.array_equal(cv[0, 0], v[0, 0, L - M:])
    for h in range(Hq):
        want = windowed_attention(q[0, h], k[0, 0], v[0, 0], B, M)
        np.testing.assert_allclose(o[0, h], want, rtol=1e-11, atol=1e-13)


def test_one_hot_selection_respects_cache_first_order_and_shared_kv_weights():
    """Slot i <- position i of [cache; block]: the first M entries are the old
    cache, so the cache never changes; swapping K and V payloads swaps results."""
    rng = np.random.default_rng(12)
    L, B, M, d = 40, 8, 8, 4
    q, k, v = rand(rng, 1, 1, L, d), rand(rng, 1, 1, L, d), rand(rng, 1, 1, L, d)
    n_steps = 4
    lo = _one_hot_logits(n_steps, 1, 1, M, B, lambda i: i)
    _, ck, cv, _ = orc.sequence_forward(q, k, v, None, B=B, M=M, logits_override=lo)
    assert np.array_equal(ck[0, 0], k[0, 0, :M]) and np.array_equal(cv[0, 0], v[0, 0, :M])
    rnd = rand(rng, n_steps, 1, 1, M, M + B, scale=2.0)
    _, ck1, cv1, _ = orc.sequence_forward(q, k, v, None, B=B, M=M, logits_override=rnd)
    _, ck2, cv2, _ = orc.sequence_forward(q, v, k, None, B=B, M=M, logits_override=rnd)
    assert np.array_equal(ck1, cv2) and np.array_equal(cv1, ck2)


def test_zero_filters_give_the_running_mean_recursion():
    """Zero filters (any bias) -> uniform weights -> every slot is the mean of
    [cache; block]:  c_n = (M c_{n-1} + sum(block_n)) / (M + B)."""
    rng = np.random.default_rng(13)
    L, B, M, d, k = 64, 8, 8, 4, 5
    q, kk, v = rand(rng, 1, 1, L, d), rand(rng, 1, 1, L, d), rand(rng, 1, 1, L, d)
    bias = rand(rng, M, scale=3.0)
    _, ck, cv, _ = orc.sequence_forward(q, kk, v, np.zeros((M, d, k)), bias, B=B, M=M)
    for src, got in ((kk[0, 0], ck[0, 0]), (v[0, 0], cv[0, 0])):
        c = src[:M].mean(0)                     # after the first compress all slots equal ...
        c = (src[:M].sum(0) + src[M:M + B].sum(0)) / (M + B)
        for n in range(2, L // B):
            c = (M * c + src[n * B:(n + 1) * B].sum(0)) / (M + B)
        np.testing.assert_allclose(got, np.tile(c, (M, 1)), rtol=1e-12, atol=1e-14)


def test_bias_shift_invariance_and_convexity():
    rng = np.random.default_rng(14)
    L, B, M, d, k = 48, 8, 8, 4, 3
    q, kk, v = rand(rng, 1, 1, L, d), rand(rng, 1, 1, L, d), rand(rng, 1, 1, L, d)
    cw = rand(rng, M, d, k)
    o1, ck1, cv1, _ = orc.sequence_forward(q, kk, v, cw, None, B=B, M=M)
    o2, ck2, cv2, _ = orc.sequence_forward(q, kk, v, cw, rand(rng, M, scale=5.0), B=B, M=M)
    np.testing.assert_allclose(o1, o2, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(ck1, ck2, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(cv1, cv2, rtol=1e-10, atol=1e-12)
    # convexity: every slot lies inside the per-channel range of the tokens seen so far
    assert np.all(ck1[0, 0] <= kk[0, 0].max(0) + 1e-12) and np.all(ck1[0, 0] >= kk[0, 0].min(0) - 1e-12)
    assert np.all(cv1[0, 0] <= v[0, 0].max(0) + 1e-12) and np.all(cv1[0, 0] >= v[0, 0].min(0) - 1e-12)


def test_one_compress_step_composed_from_library_routines():
    """A full step (conv -> softmax -> mix, cache first) rebuilt from torch
    conv1d / softmax / matmul on the explicit concatenation [cache; block]."""
    rng = np.random.default_rng(15)
    for conv_in in (0, 1):
        B, M, d, k = 6, 10, 4, 5
        L = M + B                                       # first M tokens fill (B | M not needed:
        q = rand(rng, 1, 1, L, d)                       # use len0 = M via a provided cache)
        kk, v = rand(rng, 1, 1, B, d), rand(rng, 1, 1, B, d)
        ck0, cv0 = rand(rng, 1, 1, M, d), rand(rng, 1, 1, M, d)
        C = d * (2 if conv_in else 1)
        cw, cb = rand(rng, M, C, k), rand(rng, M)
        _, ck, cv, ln = orc.sequence_forward(q[:, :, :B], kk, v, cw, cb, B=B, M=M, conv_in=conv_in,
                                             cache_k=ck0, cache_v=cv0, cache_len=M)
        YK = np.concatenate([ck0[0, 0], kk[0, 0]])
        YV = np.concatenate([cv0[0, 0], v[0, 0]])
        X = np.concatenate([YK, YV], axis=1) if conv_in else YK
        W = torch.nn.functional.conv1d(torch.from_numpy(X.T.copy())[None], torch.from_numpy(cw),
                                       torch.from_numpy(cb), padding=(k - 1) // 2)[0]
        w = torch.softmax(W, dim=1).numpy()
        assert ln == M
        np.testing.assert_allclose(ck[0, 0], w @ YK, rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(cv[0, 0], w @ YV, rtol=1e-11, atol=1e-13)


def test_partial_occupancy_and_block_larger_than_cache():
    """Cache partly full and cache + block > M: the m + B_n entries present are
    compressed; with an empty cache and B > M the block alone is compressed."""
    rng = np.random.default_rng(16)
    d, k = 4, 3
    for M, B, m0 in [(10, 7, 5), (4, 9, 0), (6, 4, 3)]:
        kk, v, q = rand(rng, 1, 1, B, d), rand(rng, 1, 1, B, d), rand(rng, 1, 1, B, d)
        ck0, cv0 = np.zeros((1, 1, M, d)), np.zeros((1, 1, M, d))
        ck0[0, 0, :m0], cv0[0, 0, :m0] = rand(rng, m0, d), rand(rng, m0, d)
        ck0[0, 0, m0:], cv0[0, 0, m0:] = 1e6, -1e6       # dead rows must never be read
        cw = rand(rng, M, d, k)
        o, ck, cv, ln = orc.sequence_forward(q, kk, v, cw, B=B, M=M, cache_k=ck0, cache_v=cv0,
                                             cache_len=m0)
        YK = np.concatenate([ck0[0, 0, :m0], kk[0, 0]])
        YV = np.concatenate([cv0[0, 0, :m0], v[0, 0]])
        W = torch.nn.functional.conv1d(torch.from_numpy(YK.T.copy())[None], torch.from_numpy(cw),
                                       padding=1)[0]
        w = torch.softmax(W, dim=1).numpy()
        assert ln == M
        np.testing.assert_allclose(ck[0, 0], w @ YK, rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(cv[0, 0], w @ YV, rtol=1e-11, atol=1e-13)
        assert np.abs(o).max() < 100                      # attention never touched the dead rows


def test_chains_are_independent_and_gqa_equals_replicated_mha():
    rng = np.random.default_rng(17)
    L, B, M, d, k, b, Hq, Hkv = 40, 8, 8, 4, 3, 2, 4, 2
    q, kk, v = rand(rng, b, Hq, L, d), rand(rng, b, Hkv, L, d), rand(rng, b, Hkv, L, d)
    cw = rand(rng, M, d, k)
    o, ck, cv, _ = orc.sequence_forward(q, kk, v, cw, B=B, M=M, nthreads=3)
    # MHA with K/V replicated per query head gives the same outputs
    g = Hq // Hkv
    o2, ck2, cv2, _ = orc.sequence_forward(q, np.repeat(kk, g, 1), np.repeat(v, g, 1), cw, B=B, M=M)
    assert np.array_equal(o, o2)
    assert np.array_equal(np.repeat(ck, g, 1), ck2) and np.array_equal(np.repeat(cv, g, 1), cv2)
    # permuting batch and kv heads permutes the results
    o3, ck3, _, _ = orc.sequence_forward(q[::-1, ::-1][:, np.r_[1, 0, 3, 2]], kk[::-1, ::-1],
                                         v[::-1, ::-1], cw, B=B, M=M)
    assert np.array_equal(o3, o[::-1, ::-1][:, np.r_[1, 0, 3, 2]])
    assert np.array_equal(ck3, ck[::-1, ::-1])
    # per-head filter banks: chain h uses bank h
    cw4 = rand(rng, Hkv, M, d, k)
    _, ck4, _, _ = orc.sequence_forward(q, kk, v, cw4, B=B, M=M)
    for h in range(Hkv):
        _, ckh, _, _ = orc.sequence_forward(q[:, h * g:(h + 1) * g], kk[:, h:h + 1], v[:, h:h + 1],
                                            cw4[h], B=B, M=M)
        assert np.array_equal(ck4[:, h:h + 1], ckh)


@pytest.mark.parametrize("mode", ["none", "f32", "bf16"])
def test_resuming_from_the_returned_cache_is_bit_identical(mode):
    rng = np.random.default_rng(18)
    L, B, M, d, k = 72, 8, 16, 4, 3
    q, kk, v = rand(rng, 1, 2, L, d), rand(rng, 1, 1, L, d), rand(rng, 1, 1, L, d)
    if mode == "bf16":
        q, kk, v = (torch.from_numpy(x).to(torch.bfloat16).double().numpy() for x in (q, kk, v))
    cw = rand(rng, M, d, k)
    o, ck, cv, ln = orc.sequence_forward(q, kk, v, cw, B=B, M=M, state_round=mode)
    for L1 in (8, 24, 40):
        oa, cka, cva, lna = orc.sequence_forward(q[:, :, :L1], kk[:, :, :L1], v[:, :, :L1], cw,
                                                 B=B, M=M, state_round=mode)
        ob, ckb, cvb, lnb = orc.sequence_forward(q[:, :, L1:], kk[:, :, L1:], v[:, :, L1:], cw,
                                                 B=B, M=M, state_round=mode, cache_k=cka,
                                                 cache_v=cva, cache_len=lna)
        assert lnb == ln
        assert np.array_equal(np.concatenate([oa, ob], 2), o)
        assert np.array_equal(ckb, ck) and np.array_equal(cvb, cv)


def test_ragged_last_segment():
    rng = np.random.default_rng(19)
    L, B, M, d, k = 45, 8, 16, 4, 3            # last block has 5 tokens
    q, kk, v = rand(rng, 1, 1, L, d), rand(rng, 1, 1, L, d), rand(rng, 1, 1, L, d)
    cw = rand(rng, M, d, k)
    o, ck, cv, _ = orc.sequence_forward(q, kk, v, cw, B=B, M=M)
    oa, cka, cva, lna = orc.sequence_forward(q[:, :, :40], kk[:, :, :40], v[:, :, :40], cw, B=B, M=M)
    YK = np.concatenate([cka[0, 0], kk[0, 0, 40:]])
    W = torch.nn.functional.conv1d(torch.from_numpy(YK.T.copy())[None], torch.from_numpy(cw),
                                   padding=1)[0]
    np.testing.assert_allclose(ck[0, 0], torch.softmax(W, 1).numpy() @ YK, rtol=1e-11, atol=1e-13)
    want_o = orc.attention_block(q[0, 0, 40:], kk[0, 0, 40:], v[0, 0, 40:], cka[0, 0], cva[0, 0])
    assert np.array_equal(o[0, 0, 40:], want_o)


# ----------------------------------------------------------------- rounding
def test_storage_rounding_matches_library_casts():
    rng = np.random.default_rng(20)
    x = np.concatenate([rng.standard_normal(5000) * 10.0 ** rng.integers(-6, 6, 5000),
                        [0.0, 1.0, -1.0, 1.00390625, 1.01171875, 3.0e-39, 1e-41]])
    bf = torch.from_numpy(x).to(torch.float32)
    # values that are exact in fp32 so a single library rounding fp32 -> bf16 is the reference
    xs = bf.double().numpy()
    want = bf.to(torch.bfloat16).double().numpy()
    got = np.array([orc.round_value(t, 2) for t in xs])
    assert np.array_equal(got, want)
    got32 = np.array([orc.round_value(t, 1) for t in x])
    assert np.array_equal(got32, torch.from_numpy(x).to(torch.float32).double().numpy())
    # a tie that double rounding through fp32 would get wrong: 1 + 2^-8 + 2^-30 is above the
    # midpoint of the bf16 neighbours 1 and 1 + 2^-7, fp32 would first drop the 2^-30
    t = 1.0 + 2.0 ** -8 + 2.0 ** -30
    assert orc.round_value(t, 2) == 1.0 + 2.0 ** -7


def test_rounded_state_stays_on_the_storage_grid():
    rng = np.random.default_rng(21)
    L, B, M, d, k = 48, 8, 8, 4, 3
    q, kk, v = (torch.from_numpy(rand(rng, 1, 1, L, d)).to(torch.bfloat16) for _ in range(3))
    cw = torch.from_numpy(rand(rng, M, d, k)).to(torch.bfloat16)
    o, ck, cv, _ = orc.sequence_forward(q, kk, v, cw, B=B, M=M, state_round="bf16")
    for t in (o, ck, cv):
        assert np.array_equal(torch.from_numpy(t).to(torch.bfloat16).double().numpy(), t)
    o64, ck64, _, _ = orc.sequence_forward(q, kk, v, cw, B=B, M=M, state_round="none")
    assert np.abs(o - o64).max() / np.abs(o64).max() < 2e-2
    assert np.abs(ck - ck64).max() / np.abs(ck64).max() < 2e-2


# ----------------------------------------------------------------- shape pin from the paper
def test_parameter_count_pins_the_filter_shape():
    """Llama-2-7B: 32 layers, 256-dimensional KV states, memory 128, width 21 ->
    about 22 million added parameters; one dense bank per layer, shared by heads."""
    with open(os.path.join(GOLDEN, "paper_parameter_count.txt")) as f:
        fields = dict(line.split("=") for line in f if "=" in line and not line.startswith("#"))
    layers, c_in, m, width = (int(fields[x]) for x in ("layers", "kv_state_dim", "memory", "width"))
    count = layers * c_in * m * width
    assert count == 22_020_096
    assert round(count / 1e6) == int(fields["added_parameters_millions"])
    assert c_in == 2 * 128                                # [K; V] of one 128-wide head


def test_scan_with_given_logits_matches_a_numpy_recursion():
    """Alg. 2 with Eq. 5's output replaced by given per-step logits: the cache
    recursion is softmax(logits_n) @ [cache; block_n], written here in numpy."""
    rng = np.random.default_rng(22)
    L, B, M, d = 40, 8, 8, 4
    q, kk, v = rand(rng, 1, 1, L, d), rand(rng, 1, 1, L, d), rand(rng, 1, 1, L, d)
    lo = rand(rng, 4, 1, 1, M, M + B, scale=2.0)
    o, ck, cv, _ = orc.sequence_forward(q, kk, v, None, B=B, M=M, logits_override=lo)
    c_k, c_v = kk[0, 0, :M].copy(), v[0, 0, :M].copy()
    for n in range(1, L // B):
        blk = slice(n * B, (n + 1) * B)
        want_o = orc.attention_block(q[0, 0, blk], kk[0, 0, blk], v[0, 0, blk], c_k, c_v)
        np.testing.assert_allclose(o[0, 0, blk], want_o, rtol=1e-10, atol=1e-13)
        w = torch.softmax(torch.from_numpy(lo[n - 1, 0, 0]), dim=1).numpy()
        c_k, c_v = w @ np.concatenate([c_k, kk[0, 0, blk]]), w @ np.concatenate([c_v, v[0, 0, blk]])
    np.testing.assert_allclose(ck[0, 0], c_k, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(cv[0, 0], c_v, rtol=1e-11, atol=1e-13)


# ---- protected slots (combination with an eviction policy)

def test_protected_slots_match_a_numpy_recursion_with_given_logits():
    """With Eq. 5's output given, the protected-slot reading written out in numpy: the softmax of
    an unprotected row runs over the unprotected cache positions and the block only, a protected
    row is carried over."""
    rng = np.random.default_rng(31)
    L, B, M, d = 48, 8, 8, 4
    q, kk, v = rand(rng, 1, 1, L, d), rand(rng, 1, 1, L, d), rand(rng, 1, 1, L, d)
    lo = rand(rng, 5, 1, 1, M, M + B, scale=2.0)
    prot = np.array([1, 0, 0, 1, 0, 0, 0, 1], dtype=bool)
    o, ck, cv, _ = orc.sequence_forward(q, kk, v, None, B=B, M=M, logits_override=lo, protect=prot)
    c_k, c_v = kk[0, 0, :M].copy(), v[0, 0, :M].copy()
    keep = np.concatenate([~prot, np.ones(B, dtype=bool)])           # positions that may carry weight
    for n in range(1, L // B):
        blk = slice(n * B, (n + 1) * B)
        want_o = orc.attention_block(q[0, 0, blk], kk[0, 0, blk], v[0, 0, blk], c_k, c_v)
        np.testing.assert_allclose(o[0, 0, blk], want_o, rtol=1e-10, atol=1e-13)   # attention sees every slot
        e = np.exp(lo[n - 1, 0, 0][:, keep] - lo[n - 1, 0, 0][:, keep].max(axis=1, keepdims=True))
        w = e / e.sum(axis=1, keepdims=True)
        new_k = w @ np.concatenate([c_k, kk[0, 0, blk]])[keep]
        new_v = w @ np.concatenate([c_v, v[0, 0, blk]])[keep]
        c_k, c_v = np.where(prot[:, None], c_k, new_k), np.where(prot[:, None], c_v, new_v)
    np.testing.assert_allclose(ck[0, 0], c_k, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(cv[0, 0], c_v, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("norm", [0, 1])
def test_protected_rows_never_change_and_an_empty_mask_changes_nothing(norm):
    rng = np.random.default_rng(32)
    b, H, L, B, M, d, kw = 2, 2, 40, 4, 8, 4, 3
    q, kk, v = rand(rng, b, H, L, d), rand(rng, b, H, L, d), rand(rng, b, H, L, d)
    cw, cb = rand(rng, M, d, kw), rand(rng, M)
    base = orc.sequence_forward(q, kk, v, cw, cb, B=B, M=M, norm=norm)
    none = orc.sequence_forward(q, kk, v, cw, cb, B=B, M=M, norm=norm, protect=np.zeros(M, bool))
    for x, y in zip(base[:3], none[:3]):
        np.testing.assert_array_equal(x, y)
    # per-chain masks: sinks (the first two tokens) on some chains, arbitrary slots on others
    prot = np.zeros((b, H, M), bool)
    prot[0, 0, :2] = True
    prot[1, 1, [3, 6]] = True
    o, ck, cv, ln = orc.sequence_forward(q, kk, v, cw, cb, B=B, M=M, norm=norm, protect=prot)
    assert ln == M
    # a protected slot still holds the token that filled it (slot i was filled by token i)
    np.testing.assert_array_equal(ck[0, 0, :2], kk[0, 0, :2])
    np.testing.assert_array_equal(cv[0, 0, :2], v[0, 0, :2])
    np.testing.assert_array_equal(ck[1, 1, [3, 6]], kk[1, 1, [3, 6]])
    # chains without protected slots are the unprotected scan, the others are not
    np.testing.assert_array_equal(ck[0, 1], base[1][0, 1])
    np.testing.assert_array_equal(o[1, 0], base[0][1, 0])
    assert np.abs(ck[0, 0, 2:] - base[1][0, 0, 2:]).max() > 1e-6
    # the unprotected rows stay convex combinations: inside the hull of everything seen
    assert ck.max() <= kk.max() + 1e-12 and ck.min() >= kk.min() - 1e-12


def test_a_fully_protected_cache_is_frozen_and_attention_still_sees_it():
    """Every slot protected: the cache stays what the first M tokens made it (sinks only), and each
    later block attends over those M tokens and itself."""
    rng = np.random.default_rng(33)
    L, B, M, d, kw = 32, 4, 8, 4, 5
    q, kk, v = rand(rng, 1, 1, L, d), rand(rng, 1, 1, L, d), rand(rng, 1, 1, L, d)
    cw = rand(rng, M, d, kw)
    o, ck, cv, _ = orc.sequence_forward(q, kk, v, cw, B=B, M=M, protect=np.ones(M, bool))
    np.testing.assert_array_equal(ck[0, 0], kk[0, 0, :M])
    np.testing.assert_array_equal(cv[0, 0], v[0, 0, :M])
    for n in range(M // B, L // B):
        blk = slice(n * B, (n + 1) * B)
        keys = np.concatenate([kk[0, 0, :M], kk[0, 0, blk]])
        vals = np.concatenate([v[0, 0, :M], v[0, 0, blk]])
        s = q[0, 0, blk] @ keys.T / np.sqrt(d)
        s[:, M:] += np.where(np.tril(np.ones((B, B), bool)), 0.0, -np.inf)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        np.testing.assert_allclose(o[0, 0, blk], (p / p.sum(axis=1, keepdims=True)) @ vals, rtol=1e-10, atol=1e-13)


def test_attention_column_sums_match_a_numpy_softmax():
    """The accumulated attention scores per cache slot (what a heavy-hitter policy ranks slots by):
    for every block, the softmax rows of all heads of the group, summed over the rows, cache
    columns only -- written out in numpy for a scan that only fills and then attends."""
    rng = np.random.default_rng(41)
    b, Hq, Hkv, L, B, M, d = 1, 4, 2, 24, 4, 8, 4
    q, kk, v = rand(rng, b, Hq, L, d), rand(rng, b, Hkv, L, d), rand(rng, b, Hkv, L, d)
    col = np.zeros((b, Hkv, M))
    prot = np.ones(M, bool)                                # frozen cache: the slots keep their meaning
    cw = rand(rng, M, d, 3)
    orc.sequence_forward(q, kk, v, cw, B=B, M=M, protect=prot, attn_colsum=col)
    want = np.zeros((b, Hkv, M))
    g = Hq // Hkv
    for n in range(L // B):
        m = min(n * B, M)                                  # live slots before block n
        blk = slice(n * B, (n + 1) * B)
        for h in range(Hq):
            keys = np.concatenate([kk[0, h // g, :m], kk[0, h // g, blk]])
            s = q[0, h, blk] @ keys.T / np.sqrt(d)
            s[:, m:] += np.where(np.tril(np.ones((B, B), bool)), 0.0, -np.inf)
            p = np.exp(s - s.max(axis=1, keepdims=True))
            p /= p.sum(axis=1, keepdims=True)
            want[0, h // g, :m] += p[:, :m].sum(axis=0)
    np.testing.assert_allclose(col, want, rtol=1e-11, atol=1e-13)
    # every query row spends at most its whole probability on the cache
    assert col.sum() <= Hq * L + 1e-9 and col.min() >= 0.0
    # accumulation: a second call adds to what is there
    before = col.copy()
    orc.sequence_forward(q, kk, v, cw, B=B, M=M, protect=prot, attn_colsum=col)
    np.testing.assert_allclose(col, 2 * before, rtol=1e-12)


# ----------------------------------------------------------------- the other reading of "a ReLU is prepended"
def test_input_side_rectifier_with_eq6_as_printed():
    """norm = 2: the rectifier acts on the convolution's input and Eq. 6 is the plain division by the
    row sum.  Pinned by the library conv1d on a rectified input, a hand-computed case, the agreement
    of the two placements where they must agree, and the guard of a vanishing row sum."""
    rng = np.random.default_rng(31)
    T, C, M, k = 23, 6, 5, 7
    X, Wc, bias = rand(rng, T, C), rand(rng, M, C, k), rand(rng, M)
    got = orc.conv_logits(X, Wc, bias, relu_input=True)
    want = torch.nn.functional.conv1d(torch.relu(torch.from_numpy(X.T.copy()))[None], torch.from_numpy(Wc),
                                      torch.from_numpy(bias), padding=(k - 1) // 2)[0].numpy()
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    assert np.abs(got - orc.conv_logits(X, Wc, bias)).max() > 0.1          # the rectifier matters
    # Eq. 6 as printed, signed entries and signed sums included
    W = rand(rng, 4, 9, scale=2.0)
    w = orc.normalise(W, norm=2)
    np.testing.assert_allclose(w, W / W.sum(1, keepdims=True), rtol=1e-13)
    np.testing.assert_allclose(w.sum(1), 1.0, rtol=0, atol=1e-12)
    # by hand: taps (1, 10, 100) on x = (1, -2, 3, -4) rectified to (1, 0, 3, 0):
    # W = (10 + 0, 1 + 300, 0 + 30, 3) = (10, 301, 30, 3), sum 344
    Wh = orc.conv_logits(np.array([[1.0], [-2.0], [3.0], [-4.0]]), np.array([[[1.0, 10.0, 100.0]]]), relu_input=True)
    assert np.array_equal(Wh, np.array([[10.0, 301.0, 30.0, 3.0]]))
    np.testing.assert_allclose(orc.normalise(Wh, norm=2), Wh / 344.0, rtol=1e-15)
    # non-negative filters and bias: the logits of a rectified input are non-negative, so rectifying
    # them again changes nothing and the two placements give the same weights (up to eps in the sum)
    Wp, bp = np.abs(Wc), np.abs(bias)
    a = orc.normalise(orc.conv_logits(X, Wp, bp, relu_input=True), norm=2)
    b = orc.normalise(orc.conv_logits(np.maximum(X, 0.0), Wp, bp), norm=1, eps=1e-12)
    np.testing.assert_allclose(a, b, rtol=1e-10)
    # a vanishing (signed) row sum is replaced by +-eps
    Wz = np.array([[1.0, -1.0, 0.0], [2.0, -2.0 - 1e-9, 0.0]])
    wz = orc.normalise(Wz, norm=2, eps=1e-6)
    np.testing.assert_allclose(wz[0], Wz[0] / 1e-6, rtol=1e-12)
    np.testing.assert_allclose(wz[1], Wz[1] / -1e-6, rtol=1e-12)


def test_one_compress_step_with_the_input_side_rectifier_composed_from_library_routines():
    """Full step with norm = 2: only the convolution's input is rectified; the entries that Eq. 4a / 4b
    fuse are the stored keys and values as they are.  Protected positions get no weight."""
    rng = np.random.default_rng(32)
    for conv_in in (0, 1):
        B, M, d, k = 6, 10, 4, 5
        q, kk, v = rand(rng, 1, 1, B, d), rand(rng, 1, 1, B, d), rand(rng, 1, 1, B, d)
        ck0, cv0 = rand(rng, 1, 1, M, d), rand(rng, 1, 1, M, d)
        C = d * (2 if conv_in else 1)
        cw, cb = np.abs(rand(rng, M, C, k)) + 0.1, np.abs(rand(rng, M))      # positive: row sums far from zero
        YK = np.concatenate([ck0[0, 0], kk[0, 0]])
        YV = np.concatenate([cv0[0, 0], v[0, 0]])
        X = np.concatenate([YK, YV], axis=1) if conv_in else YK
        W = torch.nn.functional.conv1d(torch.relu(torch.from_numpy(X.T.copy()))[None], torch.from_numpy(cw),
                                       torch.from_numpy(cb), padding=(k - 1) // 2)[0].numpy()
        for protect in (None, np.arange(M) % 4 == 1):
            _, ck, cv, ln = orc.sequence_forward(q, kk, v, cw, cb, B=B, M=M, conv_in=conv_in, norm=2,
                                                 cache_k=ck0, cache_v=cv0, cache_len=M, protect=protect)
            Wm = W.copy()
            if protect is not None:
                Wm[:, :M][:, protect] = 0.0
            w = Wm / Wm.sum(1, keepdims=True)
            nk, nv = w @ YK, w @ YV
            if protect is not None:
                nk[protect], nv[protect] = ck0[0, 0][protect], cv0[0, 0][protect]
            assert ln == M
            np.testing.assert_allclose(ck[0, 0], nk, rtol=1e-11, atol=1e-13)
            np.testing.assert_allclose(cv[0, 0], nv, rtol=1e-11, atol=1e-13)
    # forward only: the backward entry point refuses it
    with pytest.raises(ValueError):
        orc.step_backward(q, kk, v, ck0, cv0, M, cw, cb, np.zeros_like(q), np.zeros_like(ck0), np.zeros_like(cv0),
                          M=M, conv_in=conv_in, norm=2)


def test_bad_arguments_come_back_as_an_error_not_as_a_crash():
    rng = np.random.default_rng(33)
    q, kk, v = rand(rng, 1, 1, 12, 4), rand(rng, 1, 1, 12, 4), rand(rng, 1, 1, 12, 4)
    L = orc.lib()
    cfg = orc.Cfg(1, 4, 8, 3, 0, 0, 0, 0, 0.0, 1e-6)
    ln = orc.C.c_int32(0)
    dp = lambda a: a.ctypes.data_as(orc._DP)
    o, ck, cv = np.zeros_like(q), np.zeros((1, 1, 8, 4)), np.zeros((1, 1, 8, 4))
    call = lambda **kw: L.lococo_oracle_sequence_forward_protected(
        orc.C.byref(kw.get("cfg", cfg)), 1, 1, 12, kw.get("B", 4), dp(q), dp(kk), dp(v), kw.get("o", dp(o)), dp(ck),
        dp(cv), orc.C.byref(ln), kw.get("cw", None), 0, None, 0, None, None, 0, None, kw.get("nthreads", 1))
    assert call() == 1                                       # the third block compresses: filters missing
    cw = rand(rng, 8, 4, 3)
    assert call(cw=dp(cw)) == 0
    ln.value = 0
    assert call(cw=dp(cw), o=None) == 1
    assert call(cw=dp(cw), B=0) == 1
    assert call(cw=dp(cw), nthreads=0) == 1
    for bad in (dict(norm=3), dict(conv_width=4), dict(state_round=5), dict(conv_in=2), dict(norm_eps=-1.0)):
        c2 = orc.Cfg(1, 4, 8, 3, 0, 0, 0, 0, 0.0, 1e-6)
        for k_, val in bad.items():
            setattr(c2, k_, val)
        assert call(cw=dp(cw), cfg=c2) == 1, bad
    ln.value = 9
    assert call(cw=dp(cw)) == 1                              # occupancy beyond M
    with pytest.raises(ValueError):
        orc.normalise(np.zeros((2, 3)), norm=7)
    assert L.lococo_oracle_conv_logits(None, 3, 2, None, None, 2, 3, 0, None) == 1
    assert L.lococo_oracle_mix(None, None, 1, 1, 1, None) == 1
    assert L.lococo_oracle_attention_block(dp(q), dp(kk), dp(v), None, None, 2, 4, 4, 0.5, dp(o)) == 1
