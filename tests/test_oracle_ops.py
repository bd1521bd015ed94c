"""Pins of the CPU oracle's layer operations against things other than itself:
pure-Python brute force on tiny inputs, hand-evaluated Eq. 2 cases, closed
forms and the invariants the method fixes (Section 4): N=1 and stale==fresh
reproduce the full-image layer, locality of the stale rows a convolution can
see, permutation invariance and convex-hull bounds of attention.
"""
import math
import os

import numpy as np
import pytest

from df_inputs import normal
from oracle import ops

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- brute force

def brute_conv(X, w, b, stride):
    B, H, W, Cin = X.shape
    Cout = w.shape[0]
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    Y = np.zeros((B, Ho, Wo, Cout))
    for n in range(B):
        for r in range(Ho):
            for c in range(Wo):
                for o in range(Cout):
                    acc = float(b[o])
                    for ky in range(3):
                        for kx in range(3):
                            ir, ic = r * stride + ky - 1, c * stride + kx - 1
                            if 0 <= ir < H and 0 <= ic < W:
                                for i in range(Cin):
                                    acc += float(X[n, ir, ic, i]) * float(w[o, ky, kx, i])
                    Y[n, r, c, o] = acc
    return Y


def brute_attention(q, k, v, heads, scale):
    B, Lq, C = q.shape
    Lk = k.shape[1]
    d = C // heads
    out = np.zeros((B, Lq, C))
    for b in range(B):
        for h in range(heads):
            for i in range(Lq):
                logits = [scale * sum(float(q[b, i, h * d + t]) * float(k[b, j, h * d + t]) for t in range(d))
                          for j in range(Lk)]
                m = max(logits)
                e = [math.exp(x - m) for x in logits]
                z = sum(e)
                for t in range(d):
                    out[b, i, h * d + t] = sum(e[j] * float(v[b, j, h * d + t]) for j in range(Lk)) / z
    return out


@pytest.mark.parametrize("stride", [1, 2])
def test_conv_full_matches_brute_force(stride):
    X = normal(11, "X", (2, 6, 4, 3)).astype(np.float64)
    w = normal(11, "w", (5, 3, 3, 3)).astype(np.float64)
    b = normal(11, "b", (5,)).astype(np.float64)
    np.testing.assert_allclose(ops.conv3x3_full(X, w, b, stride), brute_conv(X, w, b, stride), rtol=1e-12, atol=1e-12)


def test_conv_identity_kernel_and_one_pixel():
    X = normal(12, "X", (1, 5, 7, 4)).astype(np.float64)
    w = np.zeros((4, 3, 3, 4))
    for c in range(4):
        w[c, 1, 1, c] = 1.0
    np.testing.assert_array_equal(ops.conv3x3_full(X, w, None, 1), X)
    # shift kernel: tap (0,1) reads the pixel above -> output row r equals input row r-1, first row zero
    w = np.zeros((4, 3, 3, 4))
    for c in range(4):
        w[c, 0, 1, c] = 1.0
    Y = ops.conv3x3_full(X, w, None, 1)
    np.testing.assert_array_equal(Y[:, 1:], X[:, :-1])
    np.testing.assert_array_equal(Y[:, 0], 0 * X[:, 0])
    # 1x1 image: only the centre tap can touch data
    x1 = normal(12, "x1", (1, 1, 1, 4)).astype(np.float64)
    wf = normal(12, "wf", (3, 3, 3, 4)).astype(np.float64)
    np.testing.assert_allclose(ops.conv3x3_full(x1, wf, None, 1)[0, 0, 0], wf[:, 1, 1, :] @ x1[0, 0, 0], rtol=1e-13)


@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("N,patch", [(1, 0), (2, 0), (2, 1), (4, 1), (4, 3)])
def test_conv_halo_brute_force_and_invariants(stride, N, patch):
    H, W, Cin, Cout = 8, 5 if stride == 1 else 6, 3, 4
    full = normal(13, "full", (1, H, W, Cin)).astype(np.float64)
    stale = full + 0.1 * normal(13, "noise", (1, H, W, Cin)).astype(np.float64)
    w = normal(13, "w", (Cout, 3, 3, Cin)).astype(np.float64)
    b = normal(13, "b", (Cout,)).astype(np.float64)
    R = H // N
    s, e = patch * R, (patch + 1) * R
    fresh = full[:, s:e]
    got = ops.conv3x3_halo(fresh, stale, w, b, patch, N, stride)
    # brute force on the explicitly spliced image
    X = stale.copy()
    X[:, s:e] = fresh
    np.testing.assert_allclose(got, brute_conv(X, w, b, stride)[:, s // stride:e // stride], rtol=1e-12, atol=1e-12)
    # stale == fresh: rows of the full-image output
    exact = ops.conv3x3_halo(fresh, full, w, b, patch, N, stride)
    np.testing.assert_allclose(exact, brute_conv(full, w, b, stride)[:, s // stride:e // stride], rtol=1e-12, atol=1e-12)
    if N == 1:
        np.testing.assert_array_equal(got, ops.conv3x3_full(fresh, w, b, stride))


def test_conv_halo_tiles_the_full_output_when_stale_is_fresh():
    full = normal(14, "full", (2, 8, 6, 3)).astype(np.float64)
    w = normal(14, "w", (4, 3, 3, 3)).astype(np.float64)
    b = normal(14, "b", (4,)).astype(np.float64)
    for stride in (1, 2):
        ref = ops.conv3x3_full(full, w, b, stride)
        tiles = [ops.conv3x3_halo(full[:, 2 * i:2 * i + 2], full, w, b, i, 4, stride) for i in range(4)]
        np.testing.assert_allclose(np.concatenate(tiles, axis=1), ref, rtol=1e-13, atol=1e-13)


def test_conv_halo_locality_and_linearity():
    """Only stale rows s-1 and e reach the output, and only its first/last row (stride 1)."""
    H, W, C, N, patch = 12, 5, 3, 3, 1
    s, e = 4, 8
    full = normal(15, "full", (1, H, W, C)).astype(np.float64)
    stale = normal(15, "stale", (1, H, W, C)).astype(np.float64)
    w = normal(15, "w", (4, 3, 3, C)).astype(np.float64)
    b = normal(15, "b", (4,)).astype(np.float64)
    fresh = full[:, s:e]
    base = ops.conv3x3_halo(fresh, stale, w, b, patch, N)
    far = stale.copy()
    far[:, :s - 1] += 7.0
    far[:, e + 1:] -= 5.0
    far[:, s:e] = 123.0                       # own rows of the stale buffer are never read
    np.testing.assert_array_equal(ops.conv3x3_halo(fresh, far, w, b, patch, N), base)
    near = stale.copy()
    near[:, s - 1] += 1.0
    d = ops.conv3x3_halo(fresh, near, w, b, patch, N) - base
    assert np.abs(d[:, 0]).max() > 1e-3 and np.abs(d[:, 1:]).max() == 0.0
    near = stale.copy()
    near[:, e] += 1.0
    d = ops.conv3x3_halo(fresh, near, w, b, patch, N) - base
    assert np.abs(d[:, -1]).max() > 1e-3 and np.abs(d[:, :-1]).max() == 0.0
    # linearity: conv(fresh, halo) = conv(fresh, 0) + conv(0, halo) - bias
    a = ops.conv3x3_halo(fresh, 0 * stale, w, b, patch, N)
    h = ops.conv3x3_halo(0 * fresh, stale, w, b, patch, N)
    np.testing.assert_allclose(a + h - b, base, rtol=1e-12, atol=1e-12)
    # stride 2 with an even first row: only the top halo row matters
    base2 = ops.conv3x3_halo(fresh, stale, w, b, patch, N, stride=2)
    near = stale.copy()
    near[:, e] += 1.0
    np.testing.assert_array_equal(ops.conv3x3_halo(fresh, near, w, b, patch, N, stride=2), base2)
    near = stale.copy()
    near[:, s - 1] += 1.0
    assert np.abs(ops.conv3x3_halo(fresh, near, w, b, patch, N, stride=2) - base2)[:, 0].max() > 1e-3


def test_conv_border_patches_have_zero_halo():
    H, W, C = 8, 4, 2
    full = normal(16, "full", (1, H, W, C)).astype(np.float64)
    stale = normal(16, "stale", (1, H, W, C)).astype(np.float64)
    w = normal(16, "w", (3, 3, 3, C)).astype(np.float64)
    top = ops.conv3x3_halo(full[:, :4], stale, w, None, 0, 2)
    X = np.concatenate([full[:, :4], stale[:, 4:5]], axis=1)      # no row above, one stale row below
    np.testing.assert_allclose(top, brute_conv(X, w, np.zeros(3), 1)[:, :4], rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- attention

def test_attention_dense_matches_brute_force():
    q = normal(21, "q", (2, 5, 6)).astype(np.float64)
    k = normal(21, "k", (2, 7, 6)).astype(np.float64)
    v = normal(21, "v", (2, 7, 6)).astype(np.float64)
    for heads in (1, 2, 3):
        sc = 1.0 / math.sqrt(6 // heads)
        np.testing.assert_allclose(ops.attention_dense(q, k, v, heads), brute_attention(q, k, v, heads, sc),
                                   rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("N,patch", [(1, 0), (2, 1), (4, 2)])
def test_attn_displaced_brute_force_and_invariants(N, patch):
    L, C, heads = 8, 4, 2
    Lq = L // N
    kf = normal(22, "kf", (1, L, C)).astype(np.float64)
    vf = normal(22, "vf", (1, L, C)).astype(np.float64)
    qf = normal(22, "qf", (1, L, C)).astype(np.float64)
    ks = kf + 0.3 * normal(22, "kn", (1, L, C)).astype(np.float64)
    vs = vf + 0.3 * normal(22, "vn", (1, L, C)).astype(np.float64)
    sl = slice(patch * Lq, (patch + 1) * Lq)
    got = ops.attn_displaced(qf[:, sl], kf[:, sl], vf[:, sl], ks, vs, heads, patch, N)
    K, V = ks.copy(), vs.copy()
    K[:, sl], V[:, sl] = kf[:, sl], vf[:, sl]
    sc = 1.0 / math.sqrt(C // heads)
    np.testing.assert_allclose(got, brute_attention(qf[:, sl], K, V, heads, sc), rtol=1e-12, atol=1e-13)
    # stale == fresh: rows of full self-attention
    exact = ops.attn_displaced(qf[:, sl], kf[:, sl], vf[:, sl], kf, vf, heads, patch, N)
    np.testing.assert_allclose(exact, brute_attention(qf, kf, vf, heads, sc)[:, sl], rtol=1e-12, atol=1e-13)
    # own rows of the stale buffers are never used
    ks2, vs2 = ks.copy(), vs.copy()
    ks2[:, sl] = 99.0
    vs2[:, sl] = -99.0
    np.testing.assert_array_equal(ops.attn_displaced(qf[:, sl], kf[:, sl], vf[:, sl], ks2, vs2, heads, patch, N), got)


def test_attention_properties():
    B, Lq, L, C, heads = 1, 6, 12, 8, 2
    q = normal(23, "q", (B, Lq, C)).astype(np.float64)
    k = normal(23, "k", (B, L, C)).astype(np.float64)
    v = normal(23, "v", (B, L, C)).astype(np.float64)
    o = ops.attention_dense(q, k, v, heads)
    # rows of P sum to one: with V = ones the output is ones; equal V rows are returned unchanged
    np.testing.assert_allclose(ops.attention_dense(q, k, np.ones_like(v), heads), 1.0, rtol=1e-13)
    row = normal(23, "row", (C,)).astype(np.float64)
    np.testing.assert_allclose(ops.attention_dense(q, k, np.broadcast_to(row, v.shape), heads),
                               np.broadcast_to(row, q.shape), rtol=1e-12)
    # convex hull: each output channel lies between the min and max of that channel of V
    assert (o <= v.max(axis=1, keepdims=True) + 1e-12).all() and (o >= v.min(axis=1, keepdims=True) - 1e-12).all()
    # joint permutation of K/V rows leaves the output unchanged
    perm = np.random.default_rng(0).permutation(L)
    np.testing.assert_allclose(ops.attention_dense(q, k[:, perm], v[:, perm], heads), o, rtol=1e-12, atol=1e-13)
    # zero queries: uniform attention -> mean of V
    np.testing.assert_allclose(ops.attention_dense(0 * q, k, v, heads), np.broadcast_to(v.mean(1, keepdims=True), q.shape),
                               rtol=1e-12, atol=1e-13)
    # a key far from every query (hugely negative logit) drops out: reduces to attention without it
    k2 = k.copy()
    q2 = np.abs(q) + 0.1
    k2[:, 5] = -1e4
    o_drop = ops.attention_dense(q2, k2, v, heads)
    keep = [j for j in range(L) if j != 5]
    np.testing.assert_allclose(o_drop, ops.attention_dense(q2, k2[:, keep], v[:, keep], heads), rtol=1e-12, atol=1e-13)
    # one key: output equals its value row whatever the scale
    np.testing.assert_allclose(ops.attention_dense(q, k[:, :1], v[:, :1], heads, scale=3.0),
                               np.broadcast_to(v[:, :1], q.shape), rtol=1e-13)
    # scale matters: two keys, logits l0,l1 -> weights softmax(scale*[l0,l1])
    qq = np.array([[[1.0, 0.0]]])
    kk = np.array([[[2.0, 0.0], [0.0, 0.0]]])
    vv = np.array([[[1.0, 0.0], [0.0, 1.0]]])
    p0 = math.exp(2 * 0.5) / (math.exp(2 * 0.5) + 1.0)
    np.testing.assert_allclose(ops.attention_dense(qq, kk, vv, 1, scale=0.5)[0, 0], [p0, 1 - p0], rtol=1e-13)
    # default scale is 1/sqrt(d)
    p0 = math.exp(2 / math.sqrt(2)) / (math.exp(2 / math.sqrt(2)) + 1.0)
    np.testing.assert_allclose(ops.attention_dense(qq, kk, vv, 1)[0, 0], [p0, 1 - p0], rtol=1e-13)


# ---------------------------------------------------------------- GroupNorm

def brute_groupnorm(x, gamma, beta, G, eps):
    B, H, W, C = x.shape
    cg = C // G
    y = np.zeros_like(x)
    for b in range(B):
        for g in range(G):
            vals = [float(x[b, r, c, g * cg + t]) for r in range(H) for c in range(W) for t in range(cg)]
            m = sum(vals) / len(vals)
            var = sum((u - m) ** 2 for u in vals) / len(vals)
            for r in range(H):
                for c in range(W):
                    for t in range(cg):
                        ch = g * cg + t
                        y[b, r, c, ch] = (x[b, r, c, ch] - m) / math.sqrt(var + eps) * gamma[ch] + beta[ch]
    return y


def _gn_data(seed=31, B=2, H=8, W=3, C=12):
    full = normal(seed, "full", (B, H, W, C)).astype(np.float64) * 2 + 0.5
    stale = full + 0.2 * normal(seed, "noise", (B, H, W, C)).astype(np.float64)
    gamma = normal(seed, "g", (C,)).astype(np.float64) + 1
    beta = normal(seed, "b", (C,)).astype(np.float64)
    return full, stale, gamma, beta


def test_gn_golden_hand_cases():
    rows = [l.split() for l in open(os.path.join(GOLD, "gn_eq2_hand_cases.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) == 5
    for _, mode, f0, f1, s0, q0, s1, q1, y0, y1 in rows:
        x = np.array([float(f0), float(f1)]).reshape(1, 1, 2, 1)
        st = np.array([[float(s0), float(q0)], [float(s1), float(q1)]]).reshape(2, 1, 1, 2)
        y, fs = ops.groupnorm_stale(x, st, np.ones(1), np.zeros(1), 1, 0, 2, eps=0.0, stat_mode=int(mode))
        np.testing.assert_allclose(y.ravel(), [float(y0), float(y1)], rtol=1e-14, atol=1e-15)
        np.testing.assert_allclose(fs.ravel(), [float(f0) + float(f1), float(f0) ** 2 + float(f1) ** 2], rtol=1e-15)


@pytest.mark.parametrize("N,patch", [(1, 0), (2, 0), (4, 2)])
def test_gn_sums_mode_is_groupnorm_of_the_scatter_output(N, patch):
    full, stale, gamma, beta = _gn_data()
    G, eps = 3, 1e-5
    R = full.shape[1] // N
    sl = slice(patch * R, (patch + 1) * R)
    st = ops.patch_group_sums(stale, G, N)
    y, fs = ops.groupnorm_stale(full[:, sl], st, gamma, beta, G, patch, N, eps, ops.STAT_SUMS)
    X = stale.copy()
    X[:, sl] = full[:, sl]
    np.testing.assert_allclose(y, brute_groupnorm(X, gamma, beta, G, eps)[:, sl], rtol=1e-10, atol=1e-11)
    # closed form: mean = E_stale_global + (E_fresh_local - E_stale_local) / N
    cg = full.shape[-1] // G
    n_loc = R * full.shape[2] * cg
    e_sg = st.sum(0)[..., 0] / (n_loc * N)
    e_fl = fs[..., 0] / n_loc
    e_sl = st[patch][..., 0] / n_loc
    mean_scatter = X.reshape(2, -1, G, cg).mean(axis=(1, 3))
    np.testing.assert_allclose(e_sg + (e_fl - e_sl) / N, mean_scatter, rtol=1e-12)
    if N == 1:
        for mode in (0, 1, 2):                    # with one patch only Stale GN still depends on the cache
            ym, _ = ops.groupnorm_stale(full, st, gamma, beta, G, 0, 1, eps, mode)
            np.testing.assert_allclose(ym, brute_groupnorm(full, gamma, beta, G, eps), rtol=1e-9, atol=1e-10)
        # without affine: zero mean, unit variance per group
        y0, _ = ops.groupnorm_stale(full, st, np.ones(12), np.zeros(12), G, 0, 1, 0.0)
        yg = y0.reshape(2, -1, G, cg)
        np.testing.assert_allclose(yg.mean(axis=(1, 3)), 0, atol=1e-12)
        np.testing.assert_allclose(yg.var(axis=(1, 3)), 1, rtol=1e-10)


def test_gn_all_modes_exact_when_stale_equals_fresh_and_modes_differ_otherwise():
    full, stale, gamma, beta = _gn_data(seed=32)
    G, eps, N, patch = 4, 1e-5, 4, 1
    sl = slice(2, 4)
    ref = brute_groupnorm(full, gamma, beta, G, eps)[:, sl]
    st = ops.patch_group_sums(full, G, N)
    for mode in (ops.STAT_SUMS, ops.STAT_EQ2, ops.STAT_STALE):
        y, _ = ops.groupnorm_stale(full[:, sl], st, gamma, beta, G, patch, N, eps, mode)
        np.testing.assert_allclose(y, ref, rtol=1e-9, atol=1e-10)
    # separate GN is plain GroupNorm of the patch alone
    y, _ = ops.groupnorm_stale(full[:, sl], st, gamma, beta, G, patch, N, eps, ops.STAT_SEPARATE)
    np.testing.assert_allclose(y, brute_groupnorm(full[:, sl], gamma, beta, G, eps), rtol=1e-9, atol=1e-10)
    # stale GN ignores the fresh data for its statistics
    st2 = ops.patch_group_sums(stale, G, N)
    y, _ = ops.groupnorm_stale(full[:, sl], st2, gamma, beta, G, patch, N, eps, ops.STAT_STALE)
    cg = 3
    m = stale.reshape(2, -1, G, cg).mean(axis=(1, 3))
    v = stale.reshape(2, -1, G, cg).var(axis=(1, 3))
    xg = full[:, sl].reshape(2, -1, G, cg)
    want = ((xg - m[:, None, :, None]) / np.sqrt(v[:, None, :, None] + eps)).reshape(2, 2, 3, 12) * gamma + beta
    np.testing.assert_allclose(y, want, rtol=1e-9, atol=1e-10)
    # Eq. 2 as printed: evaluate its formula independently from per-patch means
    y1, _ = ops.groupnorm_stale(full[:, sl], st2, gamma, beta, G, patch, N, eps, ops.STAT_EQ2)
    e_fl = xg.mean(axis=(1, 3))
    e_fl2 = (xg ** 2).mean(axis=(1, 3))
    sg = stale[:, sl].reshape(2, -1, G, cg)
    mean = m + (e_fl - sg.mean(axis=(1, 3)))
    m2 = (stale.reshape(2, -1, G, cg) ** 2).mean(axis=(1, 3)) + (e_fl2 - (sg ** 2).mean(axis=(1, 3)))
    var = m2 - mean ** 2
    assert (var > 0).all()
    want = ((xg - mean[:, None, :, None]) / np.sqrt(var[:, None, :, None] + eps)).reshape(2, 2, 3, 12) * gamma + beta
    np.testing.assert_allclose(y1, want, rtol=1e-9, atol=1e-10)
    y0, _ = ops.groupnorm_stale(full[:, sl], st2, gamma, beta, G, patch, N, eps, ops.STAT_SUMS)
    assert np.abs(y0 - y1).max() > 1e-4


def test_gn_silu_fusion_and_fresh_stats():
    full, stale, gamma, beta = _gn_data(seed=33)
    st = ops.patch_group_sums(stale, 3, 2)
    y, fs = ops.groupnorm_stale(full[:, :4], st, gamma, beta, 3, 0, 2)
    ys, _ = ops.groupnorm_stale(full[:, :4], st, gamma, beta, 3, 0, 2, fuse_silu=True)
    np.testing.assert_allclose(ys, y / (1 + np.exp(-y)), rtol=1e-13)
    np.testing.assert_allclose(fs, ops.patch_group_sums(full, 3, 2)[0], rtol=1e-13)
    # patch sums add up to the full-image sums
    np.testing.assert_allclose(ops.patch_group_sums(full, 3, 4).sum(0), ops.group_sums(full, 3), rtol=1e-12)


# ---------------------------------------------------------------- per-token ops, refresh

def test_scatter_and_refresh():
    full = np.arange(2 * 8 * 3, dtype=np.float64).reshape(2, 8, 3)
    fresh = -np.ones((2, 2, 3))
    out = ops.scatter(full, fresh, 2, 4)
    assert (out[:, 4:6] == -1).all() and (out[:, :4] == full[:, :4]).all() and (out[:, 6:] == full[:, 6:]).all()
    assert (full >= 0).all()                      # scatter does not modify the stale buffer
    ops.buffer_refresh(full, fresh, 2, 4)
    np.testing.assert_array_equal(full, out)
    with pytest.raises(ValueError):
        ops.scatter(full, fresh, 4, 4)
    with pytest.raises(ValueError):
        ops.scatter(full[:, :7], fresh, 0, 4)


def test_per_token_ops():
    x = normal(41, "x", (3, 5, 6)).astype(np.float64)
    w = normal(41, "w", (4, 6)).astype(np.float64)
    b = normal(41, "b", (4,)).astype(np.float64)
    y = ops.linear(x, w, b)
    for i in range(3):
        for j in range(5):
            for o in range(4):
                assert abs(y[i, j, o] - (sum(x[i, j, t] * w[o, t] for t in range(6)) + b[o])) < 1e-12
    g = normal(41, "g", (6,)).astype(np.float64)
    be = normal(41, "be", (6,)).astype(np.float64)
    ln = ops.layernorm(x, g, be, 1e-5)
    row = x[1, 2]
    m = row.mean()
    v = ((row - m) ** 2).mean()
    np.testing.assert_allclose(ln[1, 2], (row - m) / math.sqrt(v + 1e-5) * g + be, rtol=1e-12)
    # GELU: known values and the value*gelu(gate) split
    np.testing.assert_allclose(ops.gelu(np.array([0.0, 1.0, -1.0, 3.0])),
                               [0.0, 0.8413447460685429, -0.15865525393145707, 3 * 0.9986501019683699], rtol=1e-12)
    h = normal(41, "h", (2, 8)).astype(np.float64)
    np.testing.assert_allclose(ops.geglu(h), h[:, :4] * np.array([[0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in r]
                                                                  for r in h[:, 4:]]), rtol=1e-12)
    np.testing.assert_allclose(ops.silu(np.array([0.0, 1.0, -2.0])), [0.0, 1 / (1 + math.exp(-1)), -2 / (1 + math.exp(2))],
                               rtol=1e-13)
    u = ops.upsample_nearest2x(np.arange(6.0).reshape(1, 2, 3, 1))
    assert u.shape == (1, 4, 6, 1)
    np.testing.assert_array_equal(u[0, :, :, 0], [[0, 0, 1, 1, 2, 2], [0, 0, 1, 1, 2, 2], [3, 3, 4, 4, 5, 5], [3, 3, 4, 4, 5, 5]])


# ---------------------------------------------------------------- vertical strips (split_axis=2)
# Section 5.1, Baselines: the naive patch split alternates between rows and columns.  The column split is pinned by
# brute force on the explicitly spliced image, by tiling, by locality (only stale columns s-1 and e reach the output)
# and by the transposition symmetry that links it to the row split.

@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("N,patch", [(1, 0), (2, 1), (4, 0), (4, 2)])
def test_conv_halo_columns_brute_force_and_tiling(stride, N, patch):
    H, W, Cin, Cout = 5 if stride == 1 else 6, 8, 3, 4
    full = normal(41, "full", (1, H, W, Cin)).astype(np.float64)
    stale = full + 0.1 * normal(41, "noise", (1, H, W, Cin)).astype(np.float64)
    w = normal(41, "w", (Cout, 3, 3, Cin)).astype(np.float64)
    b = normal(41, "b", (Cout,)).astype(np.float64)
    Wp = W // N
    s, e = patch * Wp, (patch + 1) * Wp
    fresh = full[:, :, s:e]
    got = ops.conv3x3_halo(fresh, stale, w, b, patch, N, stride, split_axis=2)
    X = stale.copy()
    X[:, :, s:e] = fresh
    np.testing.assert_allclose(got, brute_conv(X, w, b, stride)[:, :, s // stride:e // stride], rtol=1e-12, atol=1e-12)
    # stale == fresh: the strips tile the full-image output
    tiles = [ops.conv3x3_halo(full[:, :, j * Wp:(j + 1) * Wp], full, w, b, j, N, stride, split_axis=2) for j in range(N)]
    np.testing.assert_allclose(np.concatenate(tiles, axis=2), brute_conv(full, w, b, stride), rtol=1e-12, atol=1e-12)


def test_conv_halo_columns_locality_and_transposition():
    H, W, C, N, patch = 5, 12, 3, 3, 1
    s, e = 4, 8
    full = normal(42, "full", (1, H, W, C)).astype(np.float64)
    stale = normal(42, "stale", (1, H, W, C)).astype(np.float64)
    w = normal(42, "w", (4, 3, 3, C)).astype(np.float64)
    b = normal(42, "b", (4,)).astype(np.float64)
    fresh = full[:, :, s:e]
    base = ops.conv3x3_halo(fresh, stale, w, b, patch, N, split_axis=2)
    far = stale.copy()
    far[:, :, :s - 1] += 7.0
    far[:, :, e + 1:] -= 5.0
    far[:, :, s:e] = 123.0                    # own columns of the stale buffer are never read
    np.testing.assert_array_equal(ops.conv3x3_halo(fresh, far, w, b, patch, N, split_axis=2), base)
    near = stale.copy()
    near[:, :, s - 1] += 1.0
    d = ops.conv3x3_halo(fresh, near, w, b, patch, N, split_axis=2) - base
    assert np.abs(d[:, :, 0]).max() > 1e-3 and np.abs(d[:, :, 1:]).max() == 0.0
    near = stale.copy()
    near[:, :, e] += 1.0
    d = ops.conv3x3_halo(fresh, near, w, b, patch, N, split_axis=2) - base
    assert np.abs(d[:, :, -1]).max() > 1e-3 and np.abs(d[:, :, :-1]).max() == 0.0
    # transposing image and kernel turns the column split into the row split
    t = lambda a: np.swapaxes(a, 1, 2)
    wt = np.swapaxes(w, 1, 2)
    rows = ops.conv3x3_halo(t(fresh), t(stale), wt, b, patch, N, split_axis=1)
    np.testing.assert_allclose(t(rows), base, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("N,patch", [(2, 0), (4, 3)])
def test_attn_displaced_columns_brute_force_and_invariants(N, patch):
    B, H, W, C, heads = 1, 3, 4, 4, 2
    L, Wp = H * W, W // N
    kfull = normal(43, "k", (B, L, C)).astype(np.float64)
    vfull = normal(43, "v", (B, L, C)).astype(np.float64)
    ks = kfull + 0.3 * normal(43, "kn", (B, L, C)).astype(np.float64)
    vs = vfull + 0.3 * normal(43, "vn", (B, L, C)).astype(np.float64)
    own = np.array([r * W + c for r in range(H) for c in range(patch * Wp, (patch + 1) * Wp)])   # the strip's tokens
    q = normal(43, "q", (B, len(own), C)).astype(np.float64)
    kf, vf = kfull[:, own], vfull[:, own]
    got = ops.attn_displaced(q, kf, vf, ks, vs, heads, patch, N, split_axis=2, hw=(H, W))
    K, V = ks.copy(), vs.copy()
    K[:, own], V[:, own] = kf, vf                                   # explicit splice, token by token
    np.testing.assert_allclose(got, brute_attention(q, K, V, heads, 1.0 / math.sqrt(C // heads)), rtol=1e-11, atol=1e-12)
    # the own tokens of the stale buffers are never read
    ks2, vs2 = ks.copy(), vs.copy()
    ks2[:, own], vs2[:, own] = 99.0, -99.0
    np.testing.assert_array_equal(ops.attn_displaced(q, kf, vf, ks2, vs2, heads, patch, N, split_axis=2, hw=(H, W)), got)
    # stale == fresh: rows of dense self-attention over the full map
    dense = ops.attention_dense(q, kfull, vfull, heads)
    np.testing.assert_allclose(ops.attn_displaced(q, kf, vf, kfull, vfull, heads, patch, N, split_axis=2, hw=(H, W)),
                               dense, rtol=1e-12, atol=1e-13)


def test_gn_sums_and_refresh_for_column_strips():
    B, H, W, C, G, N = 2, 4, 6, 8, 2, 3
    x = normal(44, "x", (B, H, W, C)).astype(np.float64)
    st = ops.patch_group_sums(x, G, N, axis=2)
    Wp = W // N
    for j in range(N):
        strip = x[:, :, j * Wp:(j + 1) * Wp].reshape(B, H * Wp, G, C // G)
        np.testing.assert_allclose(st[j, :, :, 0], strip.sum(axis=(1, 3)), rtol=1e-13)
        np.testing.assert_allclose(st[j, :, :, 1], (strip ** 2).sum(axis=(1, 3)), rtol=1e-13)
    np.testing.assert_allclose(st.sum(axis=0), ops.group_sums(x, G), rtol=1e-13)   # strips partition the image
    # GroupNorm of a strip with the other strips' sums = GroupNorm of the scatter output (sums mode)
    fresh = x[:, :, Wp:2 * Wp] + 0.5
    gamma, beta = np.linspace(0.5, 1.5, C), np.linspace(-1, 1, C)
    y, _ = ops.groupnorm_stale(fresh, st, gamma, beta, G, 1, N)
    X = ops.scatter(x, fresh, 1, N, axis=2)
    full, _ = ops.groupnorm_stale(X, ops.group_sums(X, G)[None], gamma, beta, G, 0, 1)
    np.testing.assert_allclose(y, full[:, :, Wp:2 * Wp], rtol=1e-11, atol=1e-12)
    d = x.copy()
    ops.buffer_refresh(d, fresh, 1, N, axis=2)
    np.testing.assert_array_equal(d, X)
