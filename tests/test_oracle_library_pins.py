"""The oracle's numpy routines against library routines of the same textbook
operations (torch CPU, float64, NCHW layout): a second, independently written
path to the same numbers."""
import numpy as np
import torch
import torch.nn.functional as F

from df_inputs import normal
from oracle import ops


def _t(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float64))


def test_conv_against_library():
    X = normal(51, "X", (2, 9, 7, 5)).astype(np.float64)
    w = normal(51, "w", (6, 3, 3, 5)).astype(np.float64)
    b = normal(51, "b", (6,)).astype(np.float64)
    for stride in (1, 2):
        ref = F.conv2d(_t(X).permute(0, 3, 1, 2), _t(w).permute(0, 3, 1, 2), _t(b), stride=stride, padding=1)
        np.testing.assert_allclose(ops.conv3x3_full(X, w, b, stride), ref.permute(0, 2, 3, 1).numpy(), rtol=1e-11, atol=1e-12)


def test_groupnorm_against_library():
    X = normal(52, "X", (2, 6, 5, 12)).astype(np.float64) * 3 + 1
    g = normal(52, "g", (12,)).astype(np.float64)
    b = normal(52, "b", (12,)).astype(np.float64)
    ref = F.group_norm(_t(X).permute(0, 3, 1, 2), 4, _t(g), _t(b), eps=1e-5).permute(0, 2, 3, 1).numpy()
    y, _ = ops.groupnorm_stale(X, ops.group_sums(X, 4)[None], g, b, 4, 0, 1, 1e-5)
    np.testing.assert_allclose(y, ref, rtol=1e-10, atol=1e-11)


def test_attention_against_library():
    q = normal(53, "q", (2, 9, 16)).astype(np.float64)
    k = normal(53, "k", (2, 11, 16)).astype(np.float64)
    v = normal(53, "v", (2, 11, 16)).astype(np.float64)
    heads = 4

    def split(a):
        return _t(a).reshape(2, -1, heads, 4).permute(0, 2, 1, 3)

    ref = F.scaled_dot_product_attention(split(q), split(k), split(v)).permute(0, 2, 1, 3).reshape(2, 9, 16).numpy()
    np.testing.assert_allclose(ops.attention_dense(q, k, v, heads), ref, rtol=1e-10, atol=1e-12)


def test_per_token_against_library():
    x = normal(54, "x", (3, 7, 10)).astype(np.float64)
    g = normal(54, "g", (10,)).astype(np.float64)
    b = normal(54, "b", (10,)).astype(np.float64)
    np.testing.assert_allclose(ops.layernorm(x, g, b, 1e-5), F.layer_norm(_t(x), (10,), _t(g), _t(b), 1e-5).numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(ops.gelu(x), F.gelu(_t(x)).numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(ops.silu(x), F.silu(_t(x)).numpy(), rtol=1e-12)
    np.testing.assert_allclose(ops.upsample_nearest2x(x[None].transpose(0, 1, 2, 3)),
                               F.interpolate(_t(x[None]).permute(0, 3, 1, 2), scale_factor=2, mode="nearest").permute(0, 2, 3, 1).numpy())
    w = normal(54, "w", (4, 10)).astype(np.float64)
    np.testing.assert_allclose(ops.linear(x, w, b[:4]), F.linear(_t(x), _t(w), _t(b[:4])).numpy(), rtol=1e-12, atol=1e-13)
