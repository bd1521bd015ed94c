"""CPU oracle of the displaced-patch layer operations (float64, numpy).

TEST INFRASTRUCTURE ONLY.  This package is the independent reference that the
HIP kernels are checked against; nothing in the product path may import it.
It shares no code with the HIP path.

Every spatially mixing layer follows the same plain definition (Section 4,
Displaced patch parallelism / Sparse operations): the device's fresh patch is
scattered into the stale full-shape activation of the previous step at its
spatial location, the ordinary full-image operator is applied to that tensor,
and the rows of the fresh region are the result.  The functions below write
exactly that: they materialise the scattered tensor, call a textbook
full-image routine and slice.  Activations are channels-last,
[B, H, W, C] (equivalently [B, L, C] with L = H*W); patches are horizontal
strips of H/N rows (split_axis=1, the default) or vertical strips of W/N
columns (split_axis=2; Section 5.1, Baselines: the naive patch split
alternates between the two directions, and nothing in Section 4 depends on the
direction).

Pins (tests/test_oracle_*.py): brute-force loops on tiny inputs, N=1 and
stale==fresh invariants, hand-evaluated Eq. 2 values (tests/golden/), locality,
linearity, permutation and convex-hull properties.  No function here is
"parity unpinned".
"""
import math

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64

STAT_SUMS = 0      # statistics of the scatter output: fresh own sums + stale sums of the other patches
STAT_EQ2 = 1       # Eq. 2 as printed: stale global + (fresh local - stale local), negative-variance fallback
STAT_SEPARATE = 2  # fresh patch only (ablation "Separate GN")
STAT_STALE = 3     # stale global only (ablation "Stale GN")


def _f64(a):
    return np.asarray(a, dtype=F64)


def patch_rows(H, patch_idx, N):
    """Row range [s, e) of patch `patch_idx` when H rows are split into N strips."""
    if H % N != 0 or not (0 <= patch_idx < N):
        raise ValueError("bad patch split")
    R = H // N
    return patch_idx * R, (patch_idx + 1) * R


def _region(shape, patch_idx, N, axis):
    """Index tuple of the patch's strip along `axis` of a [B, H, W, ...] (or [B, L, ...]) tensor."""
    s, e = patch_rows(shape[axis], patch_idx, N)
    return (slice(None),) * axis + (slice(s, e),)


def scatter(stale_full, fresh, patch_idx, N, axis=1):
    """Scatter (Section 4): copy of the stale full tensor with the fresh patch placed at its location.

    Works on [B, H, ...] tensors; the patches split `axis` (1: strips of rows, 2: strips of columns).
    """
    out = _f64(stale_full).copy()
    reg = _region(out.shape, patch_idx, N, axis)
    fresh = _f64(fresh)
    if fresh.shape != out[reg].shape:
        raise ValueError("fresh patch has the wrong shape")
    out[reg] = fresh
    return out


def buffer_refresh(dst_full, src_patch, patch_idx, N, axis=1):
    """The device's own part of the stale-buffer update (Section 4): the patch's strip <- fresh patch, in place."""
    dst_full[_region(dst_full.shape, patch_idx, N, axis)] = src_patch
    return dst_full


def silu(x):
    x = _f64(x)
    return x / (1.0 + np.exp(-x))


def gelu(x):
    """Exact (erf) GELU."""
    x = _f64(x)
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))


# ----------------------------------------------------------------------------
# convolution
# ----------------------------------------------------------------------------

def conv3x3_full(X, w, bias=None, stride=1):
    """Textbook 3x3 convolution, zero padding 1, on a full image.

    X [B,H,W,Cin], w [Cout,3,3,Cin], bias [Cout] -> [B,Ho,Wo,Cout], where output
    pixel (r, c) reads input pixels (r*stride + ky - 1, c*stride + kx - 1).
    """
    X = _f64(X)
    w = _f64(w)
    B, H, W, Cin = X.shape
    Cout = w.shape[0]
    Ho = (H + 2 - 3) // stride + 1
    Wo = (W + 2 - 3) // stride + 1
    Xp = np.zeros((B, H + 2, W + 2, Cin), dtype=F64)
    Xp[:, 1:H + 1, 1:W + 1] = X
    Y = np.zeros((B, Ho, Wo, Cout), dtype=F64)
    for ky in range(3):
        for kx in range(3):
            win = Xp[:, ky:ky + (Ho - 1) * stride + 1:stride, kx:kx + (Wo - 1) * stride + 1:stride, :]
            Y += win @ w[:, ky, kx, :].T
    if bias is not None:
        Y += _f64(bias)
    return Y


def conv3x3_halo(x_fresh, stale_full, w, bias, patch_idx, N, stride=1, act=0, split_axis=1):
    """Sparse convolution of one patch (Section 4, Sparse operations).

    The fresh strip is scattered into the stale full input, the full-image
    convolution is applied, and the output pixels of the patch are returned.
    Only the stale rows (columns, for split_axis=2) next to the patch boundary
    can influence the result.  act: 0 none, 1 SiLU.
    """
    X = scatter(stale_full, x_fresh, patch_idx, N, split_axis)
    Y = conv3x3_full(X, w, bias, stride)
    s, e = patch_rows(X.shape[split_axis], patch_idx, N)
    if s % stride or e % stride:
        raise ValueError("patch not aligned to the stride")
    out = Y[:, s // stride:e // stride] if split_axis == 1 else Y[:, :, s // stride:e // stride]
    return silu(out) if act == 1 else out


# ----------------------------------------------------------------------------
# attention
# ----------------------------------------------------------------------------

def softmax_rows(S):
    S = S - S.max(axis=-1, keepdims=True)
    P = np.exp(S)
    return P / P.sum(axis=-1, keepdims=True)


def attention_dense(q, k, v, heads, scale=None):
    """Dense multi-head softmax attention.  q [B,Lq,C], k,v [B,Lk,C], C = heads*d."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, Lq, C = q.shape
    d = C // heads
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.empty_like(q)
    for b in range(B):
        for h in range(heads):
            sl = slice(h * d, (h + 1) * d)
            P = softmax_rows((q[b, :, sl] @ k[b, :, sl].T) * scale)
            out[b, :, sl] = P @ v[b, :, sl]
    return out


def attn_displaced(q, k_fresh, v_fresh, k_stale, v_stale, heads, patch_idx, N, scale=None, split_axis=1, hw=None):
    """Self-attention turned into cross-attention (Section 4, Sparse operations).

    Queries come from the fresh tokens only; keys and values cover the whole
    feature map and are the scatter output: the patch's own tokens fresh, all
    others from the stale buffers.  q,k_fresh,v_fresh [B,Lq,C];
    k_stale,v_stale [B,L,C], tokens in row-major pixel order.  With
    split_axis=2 the patch is a strip of columns of the hw = (H, W) token
    grid: its tokens are [H, W/N] pixels in row-major order, scattered into
    columns [i*W/N, (i+1)*W/N) of every row.
    """
    if split_axis == 1:
        K = scatter(k_stale, k_fresh, patch_idx, N)
        V = scatter(v_stale, v_fresh, patch_idx, N)
    else:
        H, W = hw
        B, L, C = np.shape(k_stale)
        if L != H * W or W % N:
            raise ValueError("token grid does not match")
        K = scatter(_f64(k_stale).reshape(B, H, W, C), _f64(k_fresh).reshape(B, H, W // N, C), patch_idx, N, 2)
        V = scatter(_f64(v_stale).reshape(B, H, W, C), _f64(v_fresh).reshape(B, H, W // N, C), patch_idx, N, 2)
        K, V = K.reshape(B, L, C), V.reshape(B, L, C)
    return attention_dense(q, K, V, heads, scale)


# ----------------------------------------------------------------------------
# GroupNorm
# ----------------------------------------------------------------------------

def group_sums(x, G):
    """Per-group sum and sum of squares of a [B, R, W, C] block -> [B, G, 2]."""
    x = _f64(x)
    B = x.shape[0]
    C = x.shape[-1]
    xg = x.reshape(B, -1, G, C // G)
    return np.stack([xg.sum(axis=(1, 3)), (xg * xg).sum(axis=(1, 3))], axis=-1)


def patch_group_sums(x_full, G, N, axis=1):
    """Per-patch group sums of a full tensor: [N, B, G, 2], the content of the GroupNorm stale cache."""
    x_full = _f64(x_full)
    return np.stack([group_sums(x_full[_region(x_full.shape, j, N, axis)], G) for j in range(N)])


def groupnorm_stale(x_fresh, stale_stats, gamma, beta, G, patch_idx, N, eps=1e-5,
                    stat_mode=STAT_SUMS, fuse_silu=False):
    """Asynchronous GroupNorm of one patch (Section 4, Corrected asynchronous GroupNorm, Eq. 2).

    x_fresh [B,R,W,C]; stale_stats [N,B,G,2] per-patch (sum, sum of squares)
    cached from the previous step.  Returns (y [B,R,W,C], fresh_stats [B,G,2]).

    stat_mode
      STAT_SUMS      the statistics of the scatter output: own fresh sums plus
                     the stale sums of the other N-1 patches, over the full map.
      STAT_EQ2       Eq. 2 as printed: E[A_t] ~ E_stale_global + (E_fresh_local -
                     E_stale_local), likewise for E[A^2]; var = E[A^2] - E[A]^2;
                     groups whose variance comes out negative take the fresh
                     patch's local variance (the corrected mean is kept).
      STAT_SEPARATE  the fresh patch's own statistics.
      STAT_STALE     the stale global statistics.
    Variance is the biased one; y = (x - mean) / sqrt(var + eps) * gamma + beta.
    """
    x = _f64(x_fresh)
    st = _f64(stale_stats)
    B, R, W, C = x.shape
    cg = C // G
    n_loc = R * W * cg
    n_glob = n_loc * N
    fresh = group_sums(x, G)                                   # [B,G,2]
    loc_m, loc_m2 = fresh[..., 0] / n_loc, fresh[..., 1] / n_loc
    if stat_mode == STAT_SUMS:
        tot = fresh + st.sum(axis=0) - st[patch_idx]
        mean = tot[..., 0] / n_glob
        var = np.maximum(tot[..., 1] / n_glob - mean * mean, 0.0)
    elif stat_mode == STAT_EQ2:
        sg = st.sum(axis=0)
        mean = sg[..., 0] / n_glob + (loc_m - st[patch_idx][..., 0] / n_loc)
        m2 = sg[..., 1] / n_glob + (loc_m2 - st[patch_idx][..., 1] / n_loc)
        var = m2 - mean * mean
        var = np.where(var < 0.0, loc_m2 - loc_m * loc_m, var)
    elif stat_mode == STAT_SEPARATE:
        mean = loc_m
        var = np.maximum(loc_m2 - loc_m * loc_m, 0.0)
    elif stat_mode == STAT_STALE:
        sg = st.sum(axis=0)
        mean = sg[..., 0] / n_glob
        var = np.maximum(sg[..., 1] / n_glob - mean * mean, 0.0)
    else:
        raise ValueError("stat_mode")
    rstd = 1.0 / np.sqrt(var + eps)
    xg = x.reshape(B, R * W, G, cg)
    y = (xg - mean[:, None, :, None]) * rstd[:, None, :, None]
    y = y.reshape(B, R, W, C) * _f64(gamma) + _f64(beta)
    if fuse_silu:
        y = silu(y)
    return y, fresh


# ----------------------------------------------------------------------------
# per-token layers: applied to fresh tokens only, no cross-patch data
# (Section 4, Sparse operations; Section 5.3, Compare to tensor parallelism)
# ----------------------------------------------------------------------------

def linear(x, w, bias=None):
    """x [..., K] @ w[Nout, K]^T + bias."""
    y = _f64(x) @ _f64(w).T
    if bias is not None:
        y = y + _f64(bias)
    return y


def layernorm(x, gamma, beta, eps=1e-5):
    x = _f64(x)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * _f64(gamma) + _f64(beta)


def geglu(h):
    """h [..., 2F]: first half value, second half gate -> value * gelu(gate)."""
    h = _f64(h)
    F = h.shape[-1] // 2
    return h[..., :F] * gelu(h[..., F:])


def upsample_nearest2x(x):
    """[B,H,W,C] -> [B,2H,2W,C], each pixel repeated 2x2."""
    return np.repeat(np.repeat(_f64(x), 2, axis=1), 2, axis=2)
