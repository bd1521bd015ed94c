"""GPU parity of the layer kernels against the CPU oracle, through the C ABI.

Error metrics (gpu_util.check): relative L2 error over the whole output, 1e-5
for float32 and 2e-2 for bf16 inputs (float accumulation), plus a bound on the
worst single row (pixel / token) and on the worst single element, so that a
localised mistake cannot hide in the norm; bf16 cases feed the oracle the same
bf16-rounded inputs.  Integer-like work (the refresh copy) is bit exact.
"""
import math

import numpy as np
import pytest
import torch

import paper_2402_19481_amd as df
from df_inputs import configs, normal, round_bf16
from oracle import ops
from gpu_util import DEV, TOL_BF16, TOL_F32, check, dev, host, max_rel, rel_l2, row_err

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


# ------------------------------------------------------------------ refresh

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape,N", [((2, 8, 5, 24), 4), ((1, 64, 64, 640), 4), ((3, 6, 1, 7), 3), ((1, 4, 3, 1), 2)])
def test_buffer_refresh_bit_exact(dtype, shape, N):
    say("refresh", dtype, shape, N)
    g = torch.Generator().manual_seed(5)
    full = torch.randn(shape, generator=g).to(dtype).to(DEV)
    R = shape[1] // N
    for i in range(N):
        patch = torch.randn((shape[0], R) + shape[2:], generator=g).to(dtype).to(DEV)
        want = full.clone()
        want[:, i * R:(i + 1) * R] = patch
        got = df.buffer_refresh(full.clone(), patch, i, N)
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int16 if dtype == torch.bfloat16 else torch.int32),
                           want.view(torch.int16 if dtype == torch.bfloat16 else torch.int32))


def test_refresh_and_errors():
    x = torch.zeros(1, 8, 4, device=DEV)
    with pytest.raises(df.DfError):
        df.buffer_refresh(x, x[:, :2].contiguous(), 4, 4)          # patch index out of range
    with pytest.raises(df.DfError):
        df.buffer_refresh(torch.zeros(1, 7, 3, device=DEV), x[:, :2].contiguous(), 0, 4)   # elements not divisible
    with pytest.raises(df.DfError):
        df.groupnorm_stale(torch.zeros(1, 2, 2, 6, device=DEV), None, torch.ones(6, device=DEV),
                           torch.zeros(6, device=DEV), 4, 0, 1)     # C % G != 0
    with pytest.raises(df.DfError):
        df.attn_displaced(torch.zeros(1, 4, 48, device=DEV), torch.zeros(1, 4, 48, device=DEV),
                          torch.zeros(1, 4, 48, device=DEV), None, None, 1, 0, 1)   # head dim 48 unsupported


# ------------------------------------------------------------------ GroupNorm

def _gn_case(seed, B, H, W, C, G, N, bf16, noise=0.05, shift=0.3):
    full = normal(seed, "full", (B, H, W, C)) * 1.5 + shift
    stale = full + normal(seed, "noise", (B, H, W, C), std=noise)
    if bf16:
        full, stale = round_bf16(full), round_bf16(stale)
    gamma = normal(seed, "g", (C,), std=0.1, mean=1.0)
    beta = normal(seed, "b", (C,), std=0.1)
    st = ops.patch_group_sums(stale, G, N).astype(np.float32)
    return full, st, gamma, beta


@pytest.mark.parametrize("mode", [0, 1, 2, 3])
@pytest.mark.parametrize("silu", [False, True])
def test_groupnorm_tiny_f32_all_modes(mode, silu):
    say("gn tiny f32 mode", mode, silu)
    B, H, W, C, G, N = 1, 16, 16, 32, 8, 2
    full, st, gamma, beta = _gn_case(1, B, H, W, C, G, N, False)
    for i in range(N):
        xf = full[:, i * 8:(i + 1) * 8]
        ref, ref_fs = ops.groupnorm_stale(xf, st, gamma, beta, G, i, N, 1e-5, mode, silu)
        y, fs = df.groupnorm_stale(dev(xf), dev(st), dev(gamma), dev(beta), G, i, N, 1e-5, mode, silu)
        check(host(y), ref, False, "gn tiny patch %d" % i, say=say)
        assert rel_l2(host(fs), ref_fs) < TOL_F32


@pytest.mark.parametrize("B,H,W,C,G,N,patch,bf16", [
    (2, 9, 7, 24, 3, 3, 1, False),      # ragged pixel counts, group size 8
    (1, 12, 5, 40, 4, 4, 3, False),     # group size 10: lanes straddle groups
    (2, 8, 6, 80, 8, 2, 0, True),       # bf16, group size 10
    (1, 128, 128, 320, 32, 4, 1, True),  # configuration 3
    (1, 40, 48, 960, 32, 8, 3, True),   # widest concat input of the UNet, group size 30
    (1, 4, 4, 1280, 32, 1, 0, False),
    (1, 192, 256, 128, 32, 2, 1, True),  # two-launch path with groups narrower than a lane's 8 channels
    (2, 64, 256, 960, 32, 2, 0, True),   # the multi-step configuration's largest GroupNorm, two batch items
    (1, 96, 128, 320, 32, 2, 1, False),  # two-launch path, float32
])
def test_groupnorm_shapes(B, H, W, C, G, N, patch, bf16):
    say("gn", B, H, W, C, G, N, patch, bf16)
    full, st, gamma, beta = _gn_case(3, B, H, W, C, G, N, bf16, noise=0.02)
    R = H // N
    xf = full[:, patch * R:(patch + 1) * R]
    tol = TOL_BF16 if bf16 else TOL_F32
    for mode, silu in ((0, True), (1, False)):
        ref, ref_fs = ops.groupnorm_stale(xf, st, gamma, beta, G, patch, N, 1e-5, mode, silu)
        y, fs = df.groupnorm_stale(dev(xf, bf16), dev(st), dev(gamma), dev(beta), G, patch, N, 1e-5, mode, silu)
        check(host(y), ref, bf16, "gn mode %d" % mode, say=say)
        assert rel_l2(host(fs), ref_fs) < 1e-5


@pytest.mark.parametrize("R,W,C,G,N,patch", [
    (8, 16, 64, 8, 2, 1),        # one launch, pixels held in registers
    (32, 128, 64, 4, 4, 2),      # one launch per group, two passes over the patch
    (64, 128, 64, 4, 2, 0),      # statistics / finalize / apply kernels
])
@pytest.mark.parametrize("mode", [0, 1])
def test_groupnorm_mean_far_from_zero_f32(R, W, C, G, N, patch, mode):
    """Activations whose mean is 50 standard deviations away from zero: E[x^2] - E[x]^2 of plain float sums would lose
    2500 ulps and miss the float32 tolerance; the kernels sum x minus a pivot and combine in double."""
    say("gn mean = 50 sigma", R, W, C, G, N, patch, mode)
    H = R * N
    full = (normal(9, "full", (1, H, W, C)) + 50.0).astype(np.float32)
    stale = (full + normal(9, "noise", (1, H, W, C), std=0.05)).astype(np.float32)
    gamma, beta = normal(9, "g", (C,), std=0.1, mean=1.0), normal(9, "b", (C,), std=0.1)
    st = ops.patch_group_sums(stale, G, N).astype(np.float32)
    xf = full[:, patch * R:(patch + 1) * R]
    ref, ref_fs = ops.groupnorm_stale(xf, st, gamma, beta, G, patch, N, 1e-5, mode, False)
    y, fs = df.groupnorm_stale(dev(xf), dev(st), dev(gamma), dev(beta), G, patch, N, 1e-5, mode, False)
    check(host(y), ref, False, "gn mean=50sigma mode %d" % mode, say=say)
    assert rel_l2(host(fs), ref_fs) < 1e-6
    # the plain formula in float32 is indeed outside the tolerance here (what the test guards against)
    x32 = xf.reshape(1, R * W, G, C // G)
    m32 = x32.mean(axis=(1, 3), dtype=np.float32)
    v32 = (x32 * x32).mean(axis=(1, 3), dtype=np.float32) - m32 * m32
    say("   plain float32 variance is off by", float(np.abs(v32 / x32.var(axis=(1, 3), dtype=np.float64) - 1).max()))


def test_groupnorm_negative_variance_fallback_and_in_place_stats():
    # own stale slot with a huge second moment drives Eq. 2's variance negative
    B, R, W, C, G, N = 1, 4, 4, 8, 2, 2
    x = normal(7, "x", (B, R, W, C), std=0.1, mean=1.0)
    st = np.zeros((N, B, G, 2), dtype=np.float32)
    st[0, :, :, 1] = 1e4
    gamma, beta = np.ones(C, np.float32), np.zeros(C, np.float32)
    ref, ref_fs = ops.groupnorm_stale(x, st, gamma, beta, G, 0, N, 1e-5, ops.STAT_EQ2)
    st_d = dev(st)
    y, fs = df.groupnorm_stale(dev(x), st_d, dev(gamma), dev(beta), G, 0, N, 1e-5, df.GN_EQ2,
                               fresh_stats_out=st_d[0])
    assert rel_l2(host(y), ref) < 1e-4
    np.testing.assert_allclose(host(st_d)[0], ref_fs, rtol=1e-5)      # refreshed in place after being read
    np.testing.assert_array_equal(host(st_d)[1], st[1])


# ------------------------------------------------------------------ convolution

def _conv_case(seed, B, H, W, Cin, Cout, bf16, noise=0.5):
    full = normal(seed, "full", (B, H, W, Cin))
    stale = full + normal(seed, "noise", (B, H, W, Cin), std=noise)
    w = normal(seed, "w", (Cout, 3, 3, Cin), std=1.0 / math.sqrt(9 * Cin))
    b = normal(seed, "b", (Cout,), std=0.1)
    if bf16:
        full, stale, w = round_bf16(full), round_bf16(stale), round_bf16(w)
    return full, stale, w, b


@pytest.mark.parametrize("B,H,W,Cin,Cout,N,stride,bf16", [
    (1, 16, 16, 32, 32, 2, 1, False),    # configuration 1
    (2, 12, 6, 5, 7, 3, 1, False),       # odd channel counts
    (1, 16, 8, 8, 12, 4, 2, False),      # stride 2
    (1, 8, 8, 4, 64, 2, 1, True),        # conv_in-like: 4 input channels (direct kernel)
    (1, 8, 8, 128, 4, 2, 1, True),       # conv_out-like: 4 output channels (wave kernel)
    (2, 16, 12, 64, 96, 4, 1, True),     # MFMA tile path, ragged M and N tiles
    (1, 16, 24, 96, 64, 4, 2, True),     # MFMA, stride 2
    (1, 32, 40, 64, 320, 2, 1, True),    # MFMA, several N tiles
])
def test_conv_halo_all_patches(B, H, W, Cin, Cout, N, stride, bf16):
    say("conv", B, H, W, Cin, Cout, N, stride, bf16)
    full, stale, w, b = _conv_case(11, B, H, W, Cin, Cout, bf16)
    R = H // N
    tol = TOL_BF16 if bf16 else TOL_F32
    for i in range(N):
        xf = full[:, i * R:(i + 1) * R]
        for act in (0, 1):
            ref = ops.conv3x3_halo(xf, stale, w, b, i, N, stride, act)
            y = df.conv3x3_halo(dev(xf, bf16), dev(stale, bf16), dev(w, bf16), dev(b), i, N, stride, act)
            check(host(y), ref, bf16, "conv patch %d act %d" % (i, act), say=say)
    # one patch: the full-image convolution, no stale buffer needed
    ref = ops.conv3x3_full(full, w, b, stride)
    y = df.conv3x3_halo(dev(full, bf16), None, dev(w, bf16), dev(b), 0, 1, stride, 0)
    check(host(y), ref, bf16, "conv N=1", say=say)


def test_conv_config3_full_size():
    t = configs.conv_gn_stage()
    m = t["meta"]
    N, R = m["N"], m["H"] // m["N"]
    say("conv cfg3", m)
    for i in (0, 1, 3):
        xf = t["x_full"][:, i * R:(i + 1) * R]
        ref = ops.conv3x3_halo(xf, t["x_stale"], t["conv_w"], t["conv_b"], i, N, 1, 1)
        y = df.conv3x3_halo(dev(xf, True), dev(t["x_stale"], True), dev(t["conv_w"], True), dev(t["conv_b"]), i, N, 1, 1)
        check(host(y), ref, True, "conv cfg3 patch %d" % i, say=say)


# ------------------------------------------------------------------ attention

def _attn_case(seed, B, L, C, N, patch, bf16, stale_std=0.5):
    Lq = L // N
    rnd = round_bf16 if bf16 else (lambda a: a)
    kfull = normal(seed, "k", (B, L, C))
    vfull = normal(seed, "v", (B, L, C))
    sl = slice(patch * Lq, (patch + 1) * Lq)
    return dict(q=rnd(normal(seed, "q", (B, Lq, C))), kf=rnd(kfull[:, sl].copy()), vf=rnd(vfull[:, sl].copy()),
                ks=rnd(kfull + normal(seed, "kn", (B, L, C), std=stale_std)),
                vs=rnd(vfull + normal(seed, "vn", (B, L, C), std=stale_std)))


@pytest.mark.parametrize("B,L,C,heads,N,patch,bf16", [
    (1, 256, 32, 1, 2, 0, False),       # configuration 1
    (2, 96, 128, 2, 3, 1, False),       # d = 64 in float32, fewer keys than two waves' stride
    (1, 512, 128, 2, 4, 2, True),       # bf16 MFMA kernel
    (2, 600, 64, 1, 4, 3, True),        # ragged: 150 queries, 600 keys (partial tiles), batch 2
    (1, 2400, 192, 3, 8, 5, True),      # level-2 shape of the 1280x1920 share: 300 queries, split keys
    (1, 77 * 1, 128, 2, 1, 0, True),    # 77 keys, everything fresh (cross-attention shape)
])
def test_attention_displaced(B, L, C, heads, N, patch, bf16):
    say("attn", B, L, C, heads, N, patch, bf16)
    t = _attn_case(21, B, L, C, N, patch, bf16)
    ref = ops.attn_displaced(t["q"], t["kf"], t["vf"], t["ks"], t["vs"], heads, patch, N)
    o = df.attn_displaced(dev(t["q"], bf16), dev(t["kf"], bf16), dev(t["vf"], bf16), dev(t["ks"], bf16),
                          dev(t["vs"], bf16), heads, patch, N)
    check(host(o), ref, bf16, "attn", say=say)
    # own rows of the stale buffers must not be read
    ks2, vs2 = t["ks"].copy(), t["vs"].copy()
    Lq = L // N
    ks2[:, patch * Lq:(patch + 1) * Lq] = 50.0
    vs2[:, patch * Lq:(patch + 1) * Lq] = -50.0
    o2 = df.attn_displaced(dev(t["q"], bf16), dev(t["kf"], bf16), dev(t["vf"], bf16), dev(ks2, bf16), dev(vs2, bf16),
                           heads, patch, N)
    np.testing.assert_array_equal(host(o2), host(o))


def test_attention_config2_full_size():
    t = configs.attn_core()
    m = t["meta"]
    say("attn cfg2", m)
    ref = ops.attn_displaced(t["q"], t["k_fresh"], t["v_fresh"], t["k_stale"], t["v_stale"], m["heads"],
                             m["patch_idx"], m["N"])
    o = df.attn_displaced(dev(t["q"], True), dev(t["k_fresh"], True), dev(t["v_fresh"], True), dev(t["k_stale"], True),
                          dev(t["v_stale"], True), m["heads"], m["patch_idx"], m["N"])
    check(host(o), ref, True, "attn cfg2", say=say)


def test_attention_large_logits_are_stable():
    # scaled-up queries: softmax close to one-hot, needs the running-max rescaling
    t = _attn_case(22, 1, 512, 64, 2, 1, True)
    q = round_bf16(t["q"] * 6.0)
    ref = ops.attn_displaced(q, t["kf"], t["vf"], t["ks"], t["vs"], 1, 1, 2)
    o = df.attn_displaced(dev(q, True), dev(t["kf"], True), dev(t["vf"], True), dev(t["ks"], True), dev(t["vs"], True),
                          1, 1, 2)
    check(host(o), ref, True, "attn large logits", say=say)


# ------------------------------------------------------------------ configuration 1 block

def test_tiny_block_chain_f32():
    """GroupNorm -> conv3x3 -> single-head attention on patch 0 of 2, stale buffers left by a
    full-image pass of the same block over the stale input (all through the oracle)."""
    t = configs.tiny_block()
    m = t["meta"]
    H, W, C, N, G = m["H"], m["W"], m["C"], m["N"], m["G"]
    x, xs = t["x_full"], t["x_full"] + t["stale_noise"]
    # full-image pass on the stale input defines the three stale buffers
    gn_s, _ = ops.groupnorm_stale(xs, ops.group_sums(xs, G)[None], t["gamma"], t["beta"], G, 0, 1, m["eps"])
    st_stats = ops.patch_group_sums(xs, G, N).astype(np.float32)
    conv_s = ops.conv3x3_full(gn_s, t["conv_w"], t["conv_b"])
    kv_s = conv_s.reshape(1, H * W, C)
    for i in range(N):
        R = H // N
        xf = x[:, i * R:(i + 1) * R]
        r1, _ = ops.groupnorm_stale(xf, st_stats, t["gamma"], t["beta"], G, i, N, m["eps"])
        r2 = ops.conv3x3_halo(r1, gn_s, t["conv_w"], t["conv_b"], i, N)
        tok = r2.reshape(1, R * W, C)
        r3 = ops.attn_displaced(tok, tok, tok, kv_s, kv_s, 1, i, N)
        g1, _ = df.groupnorm_stale(dev(xf), dev(st_stats), dev(t["gamma"]), dev(t["beta"]), G, i, N, m["eps"])
        g2 = df.conv3x3_halo(g1, dev(gn_s), dev(t["conv_w"]), dev(t["conv_b"]), i, N)
        gt = g2.reshape(1, R * W, C)
        g3 = df.attn_displaced(gt, gt, gt, dev(kv_s), dev(kv_s), 1, i, N)
        for nm, g, r in (("gn", g1, r1), ("conv", g2, r2), ("attn", g3, r3.reshape(1, R * W, C))):
            check(host(g), r.reshape(host(g).shape), False, "tiny block patch %d %s" % (i, nm), say=say)


# ------------------------------------------------------------------ linear layers (per-token, fresh rows only)

@pytest.mark.parametrize("M,N,K,out_f32,res", [
    (300, 1280, 1280, True, True),     # level-2 projection of the 1280x1920 share: few tiles, split along K
    (300, 1280, 5120, True, True),     # feed-forward output: deep K
    (300, 3840, 1280, False, False),   # fused QKV
    (77, 2560, 2048, False, False),    # text K/V projection: ragged rows
    (1200, 640, 2560, True, True),
    (1, 320, 1280, True, False),       # embedding projection: a single row
    (130, 192, 96, False, False),      # K not a multiple of 64: register-staged kernel
    (4800, 320, 960, True, False),     # 1x1 shortcut convolution
])
def test_linear(M, N, K, out_f32, res):
    say("linear", M, N, K, out_f32, res)
    x = round_bf16(normal(31, "x", (M, K)))
    w = round_bf16(normal(31, "w", (N, K), std=1.0 / math.sqrt(K)))
    b = normal(31, "b", (N,), std=0.1)
    r = normal(31, "r", (M, N)) if res else None
    ref = ops.linear(x, w, b) + (r if res else 0.0)
    y = df.linear(dev(x, True), dev(w, True), dev(b), dev(r) if res else None,
                  out_dtype=torch.float32 if out_f32 else torch.bfloat16)
    # float output of bf16 operands: the only rounding is the float accumulation order
    check(host(y), ref, True, "linear", tol=(2e-3 if out_f32 else TOL_BF16), row_tol=(4e-3 if out_f32 else None),
          elt_tol=(4e-3 if out_f32 else None), say=say)
    if res and out_f32:                 # in-place residual: out aliases the residual
        rd = dev(r)
        df.linear(dev(x, True), dev(w, True), dev(b), rd, out=rd)
        assert rel_l2(host(rd), ref) < 2e-3
    # run-to-run determinism (split-K partials are added in a fixed order)
    y2 = df.linear(dev(x, True), dev(w, True), dev(b), dev(r) if res else None,
                   out_dtype=torch.float32 if out_f32 else torch.bfloat16)
    np.testing.assert_array_equal(host(y), host(y2))


# ---------------------------------------------------------------------------------------------------------------
# linear layers on fragment-packed operands
# ---------------------------------------------------------------------------------------------------------------

def unpack_rows(packed, M, K):
    """Decodes the packed layout documented in include/distrifusion.h: fragments [ceil(M/32)][K/16][64][8]; slot l of
    fragment (rt, kf) holds row rt*32 + l%32, columns kf*16 + 8*(l/32) .. +7."""
    MT, KF = (M + 31) // 32, K // 16
    a = packed.reshape(MT, KF, 2, 32, 8)                 # [rt, kf, l/32, l%32, e]
    full = a.transpose(0, 3, 1, 2, 4).reshape(MT * 32, K)
    return full[:M], full[M:]


def test_pack_rows_layout():
    M, K = 77, 96
    say("pack_rows", M, K)
    x = round_bf16(normal(40, "x", (M, K)))
    p = host(df.pack_rows(dev(x, True)))
    got, pad = unpack_rows(p, M, K)
    np.testing.assert_array_equal(got, x)
    assert not pad.any()                                 # rows beyond M are zero


@pytest.mark.parametrize("M,N,K,variant", [
    (300, 1280, 1280, "plain"),        # level-2 projection of the patch step, 10 ragged token fragments
    (300, 1280, 5120, "plain"),        # feed-forward output (deep K)
    (77, 64, 128, "plain"),            # fewer k-steps per wave than the prefetch depth
    (33, 96, 192, "plain"),            # odd number of 32-feature fragments
    (300, 384, 256, "ln"),             # LayerNorm folded into the layer
    (300, 2560, 320, "geglu"),         # value * gelu(gate)
    (130, 512, 128, "ln_geglu"),
    (1200, 640, 640, "plain"),
    (300, 3840, 1280, "ln"),           # 64 x 96 wave tile: a single round of workgroups, reduced row by row
    (300, 10240, 1280, "ln_geglu"),    # 128 x 128 wave tile (two value / gate fragment pairs), ragged third row group
    (270, 1024, 1024, "geglu"),        # 128 x 128 tile without the folded norm; 9 token fragments
    (270, 3840, 1280, "plain"),        # 64 x 96 tile, odd number of token fragments (last row group half empty)
    (300, 1280, 1280, "ln_far"),       # folded LayerNorm on rows whose mean is 50 standard deviations from zero
])
def test_linear_packed(M, N, K, variant):
    say("linear_packed", M, N, K, variant)
    x = round_bf16(normal(41, "x", (M, K)) + (50.0 if "far" in variant else 0.3))
    w = round_bf16(normal(41, "w", (N, K), std=1.0 / math.sqrt(K)))
    b = normal(41, "b", (N,), std=0.1)
    geglu = "geglu" in variant
    No = N // 2 if geglu else N
    r = normal(41, "r", (M, No))
    xp = df.pack_rows(dev(x, True))
    if "ln" in variant:
        gamma = 1.0 + 0.2 * normal(41, "g", (K,))
        beta = 0.1 * normal(41, "be", (K,))
        pre = ops.linear(ops.layernorm(x, gamma, beta, 1e-5), w, b)
        # host-side fold in float64 from the bf16-rounded scaled weights, as the header defines it
        wg = round_bf16(w * gamma[None, :].astype(np.float32))
        ln_s = wg.astype(np.float64).sum(1)
        ln_t = w.astype(np.float64) @ beta.astype(np.float64) + b
        wp = df.pack_linear_weight(dev(w, True), dev(gamma.astype(np.float32)))
        kw = dict(ln_s=dev(ln_s.astype(np.float32)), ln_t=dev(ln_t.astype(np.float32)), ln_eps=1e-5)
    else:
        pre = ops.linear(x, w, b)
        wp = df.pack_linear_weight(dev(w, True))
        kw = dict(bias=dev(b))
    ref = ops.geglu(pre) if geglu else pre
    ref = ref + r
    rd = dev(r)
    outs = df.linear_packed(xp, wp, M, N, K, residual=rd, geglu=geglu, want=("f32", "packed", "rows"), **kw)
    tol32 = 1e-2 if "ln" in variant else 2e-3           # folded norm: weights rounded after scaling by gamma
    check(host(outs["f32"]), ref, True, "linear_packed f32", tol=tol32, row_tol=4 * tol32, elt_tol=4 * tol32, say=say)
    check(host(outs["rows"]), ref, True, "linear_packed rows", say=say)
    got, _ = unpack_rows(host(outs["packed"]), M, No)
    np.testing.assert_array_equal(got, host(outs["rows"]))       # both bf16 outputs round the same float
    # determinism and in-place residual
    outs2 = df.linear_packed(xp, wp, M, N, K, residual=rd, geglu=geglu, want=("f32",), **kw)
    np.testing.assert_array_equal(host(outs["f32"]), host(outs2["f32"]))


def test_geglu_gate_function_pointwise():
    """The kernels' GELU against the erf definition, value by value: identity weights turn the GEGLU layer into
    out[m, f] = x[m, f] * gelu(x[m, f]) with exact products, on a grid of bf16-representable arguments."""
    say("geglu pointwise")
    M, F = 256, 64
    grid = (np.arange(M * F, dtype=np.float64) % 257 - 128.0) / 16.0          # -8 .. 8 in steps of 1/16
    x = round_bf16(grid.reshape(M, F).astype(np.float32))
    assert np.array_equal(x, grid.reshape(M, F).astype(np.float32))
    eye = np.eye(F, dtype=np.float32)
    w = np.concatenate([eye, eye], 0)                                          # value rows, then gate rows
    xp = df.pack_rows(dev(x, True))
    wp = df.pack_linear_weight(dev(w, True))
    out = host(df.linear_packed(xp, wp, M, 2 * F, F, geglu=True, want=("f32",))["f32"]).astype(np.float64)
    xd = x.astype(np.float64)
    erf = np.vectorize(math.erf)
    ref = xd * (0.5 * xd * (1.0 + erf(xd / math.sqrt(2.0))))
    err = np.abs(out - ref)
    say("   max abs err", err.max())
    assert (err <= 4e-6 * np.maximum(1.0, xd * xd)).all()


# ---------------------------------------------------------------------------------------------------------------
# the attention forms of the UNet step: transposed values in the stale buffer; cross-attention fused into its
# query projection
# ---------------------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("B,Lq,L,heads,packed", [
    (1, 300, 2400, 20, True),       # level 2 of the benchmark step: ragged last key tile, 2.3 query blocks
    (1, 1200, 9600, 10, False),     # level 1
    (2, 96, 200, 2, True),          # two batch items, key count not a multiple of 8
    (1, 33, 64, 1, False),          # a single full tile, ragged queries: the second wave group has no keys
    (1, 40, 600, 2, False),         # key ranges rounded up to 128: fewer ranges than first chosen, last one ragged
    (1, 130, 1100, 3, True),        # odd number of 64-key tiles in a range: the second group's last tile is missing
    (2, 300, 2400, 4, True),        # two batch items in the form whose waves split the keys (80 workgroups)
    (2, 300, 2400, 20, True),       # two batch items of the benchmark level: 400 blocks, so split key ranges in the two-group kernel
    (1, 4096, 8192, 10, False),     # > 600 workgroups: the single-group, three-stage form
    (1, 512, 4096, 2, False),       # the largest query count of the form whose waves split the keys
    (2, 70, 1003, 3, False),        # that form: ragged queries, 11 valid keys in the last tile, two batch items
    (1, 300, 515, 1, True),         # that form: 9 tiles on 8 waves, 3 valid keys in the last tile
    (1, 32, 512, 1, True),          # that form: one tile per wave
])
def test_attn_stale_vt(B, Lq, L, heads, packed):
    say("attn_stale_vt", B, Lq, L, heads, packed)
    C = heads * 64
    q = round_bf16(normal(51, "q", (B, Lq, C)))
    k = round_bf16(normal(51, "k", (B, L, C)))
    v = round_bf16(normal(51, "v", (B, L, C)))
    ref = ops.attention_dense(q, k, v, heads)
    Lp = (L + 63) // 64 * 64
    vt = np.full((B, C, Lp), np.nan, dtype=np.float32)      # pad columns hold NaN: they must never contribute
    vt[:, :, :L] = v.transpose(0, 2, 1)
    vt_d = dev(np.nan_to_num(vt, nan=0.0), True)
    if Lp > L:
        vt_d[:, :, L:] = float("nan")
    out = df.attn_stale_vt(dev(q, True), dev(k, True), vt_d, heads, L, packed=packed)
    got = unpack_rows(host(out), B * Lq, C)[0].reshape(B, Lq, C) if packed else host(out)
    check(got, ref, True, "attn_stale_vt", say=say)
    out2 = df.attn_stale_vt(dev(q, True), dev(k, True), vt_d, heads, L, packed=packed)
    got2 = unpack_rows(host(out2), B * Lq, C)[0].reshape(B, Lq, C) if packed else host(out2)
    np.testing.assert_array_equal(got, got2)            # reproducible (padding rows of a packed output are not written)


@pytest.mark.parametrize("B,rows,C,TL,count,block", [
    (1, 300, 1280, 77, 3, 1),       # level 2 of the benchmark step
    (1, 1200, 640, 77, 2, 0),       # level 1
    (2, 64, 128, 13, 2, 1),         # two batch items, one key tile
    (1, 40, 256, 128, 1, 0),        # the longest supported text
])
def test_cross_attn_packed(B, rows, C, TL, count, block):
    say("cross_attn_packed", B, rows, C, TL, count, block)
    heads = C // 64
    M = B * rows
    x = round_bf16(normal(52, "x", (M, C)) + 0.2)
    wq = round_bf16(normal(52, "wq", (C, C), std=1.0 / math.sqrt(C)))
    gamma = (1.0 + 0.2 * normal(52, "g", (C,))).astype(np.float32)
    beta = (0.1 * normal(52, "be", (C,))).astype(np.float32)
    kv = round_bf16(normal(52, "kv", (B * TL, count * 2 * C)))
    qref = ops.linear(ops.layernorm(x, gamma, beta, 1e-5), wq).reshape(B, rows, C)
    kref = kv[:, block * 2 * C:block * 2 * C + C].reshape(B, TL, C)
    vref = kv[:, block * 2 * C + C:(block + 1) * 2 * C].reshape(B, TL, C)
    ref = ops.attention_dense(qref, kref, vref, heads).reshape(M, C)
    wg = round_bf16(wq * gamma[None, :])
    ln_s = wg.astype(np.float64).sum(1)
    ln_t = wq.astype(np.float64) @ beta.astype(np.float64)
    xp = df.pack_rows(dev(x, True))
    wp = df.pack_linear_weight(dev(wq, True), dev(gamma))
    kvp = df.pack_text_kv(dev(kv, True), B, TL, count, C)
    out = df.cross_attn_packed(xp, wp, dev(ln_s.astype(np.float32)), dev(ln_t.astype(np.float32)), kvp, B, rows, C, TL,
                               count, block)
    got = unpack_rows(host(out), M, C)[0]
    check(got, ref, True, "cross_attn_packed", say=say)


# ---------------------------------------------------------------------------------------------------------------
# chains of the benchmark configurations through the per-operation entry points
# ---------------------------------------------------------------------------------------------------------------

def test_config2_self_and_cross_attention_layer():
    """Configuration 2 as a whole layer: LayerNorm + fused Q/K/V projection of the patch's 1024 tokens, displaced
    self-attention against 3072 stale + 1024 fresh key rows, output projection with residual, then LayerNorm + query
    projection + cross-attention to the 77 text tokens and its output projection.  The stale K/V are the projections of
    the full hidden state plus 0.02 N(0,1) (added in K/V space), rounded to bf16 once and given to both sides."""
    t = configs.attn_layer()
    m = t["meta"]
    L, C, N, heads, TL = m["L"], m["C"], m["N"], m["heads"], m["text_len"]
    Lq, patch = L // N, 1
    say("cfg2 layer", m)
    rows = slice(patch * Lq, (patch + 1) * Lq)
    hid = t["hidden"][0]                                                  # [L, C], bf16-representable
    # oracle: stale buffers from the full hidden state, then the patch's chain
    n1 = ops.layernorm(hid, t["ln1_g"], t["ln1_b"])
    kv_full = ops.linear(n1, t["qkv_w"][C:])
    k_stale = round_bf16((kv_full[:, :C] + t["k_noise"][0]).astype(np.float32))[None]
    v_stale = round_bf16((kv_full[:, C:] + t["v_noise"][0]).astype(np.float32))[None]
    qkv = ops.linear(n1[rows], t["qkv_w"])
    a1 = ops.attn_displaced(qkv[None, :, :C], qkv[None, :, C:2 * C], qkv[None, :, 2 * C:], k_stale, v_stale, heads,
                            patch, N)[0]
    h1 = hid[rows] + ops.linear(a1, t["o_w"], t["o_b"])
    n2 = ops.layernorm(h1, t["ln2_g"], t["ln2_b"])
    kv2 = ops.linear(t["text"][0], t["kv2_w"])
    a2 = ops.attention_dense(ops.linear(n2, t["q2_w"])[None], kv2[None, :, :C], kv2[None, :, C:], heads)[0]
    ref = h1 + ops.linear(a2, t["o2_w"], t["o2_b"])

    # GPU: every arithmetic step through the C ABI (torch only slices and re-types buffers)
    def fold(w, gamma, beta):
        wg = round_bf16(w * gamma[None, :].astype(np.float32))
        return (df.pack_linear_weight(dev(w, True), dev(gamma.astype(np.float32))),
                dev(wg.astype(np.float64).sum(1).astype(np.float32)),
                dev((w.astype(np.float64) @ beta.astype(np.float64)).astype(np.float32)))
    hp = df.pack_rows(dev(hid[rows], True))
    wq, s1, t1 = fold(t["qkv_w"], t["ln1_g"], t["ln1_b"])
    qkv_d = df.linear_packed(hp, wq, Lq, 3 * C, C, ln_s=s1, ln_t=t1, want=("rows",))["rows"]
    q_d, k_d, v_d = (qkv_d[:, j * C:(j + 1) * C].contiguous().view(1, Lq, C) for j in range(3))
    a1_d = df.attn_displaced(q_d, k_d, v_d, dev(k_stale, True), dev(v_stale, True), heads, patch, N)
    check(host(a1_d)[0], a1, True, "cfg2 self-attention output", say=say)
    hid_f = dev(hid[rows])
    h1_d = df.linear(a1_d.view(Lq, C), dev(t["o_w"], True), dev(t["o_b"]), hid_f, out_dtype=torch.float32)
    check(host(h1_d), h1, True, "cfg2 hidden after self-attention", say=say)
    h1_b = torch.empty(Lq, C, dtype=torch.bfloat16, device=DEV)          # the same layer again with a bf16 result:
    df.linear(a1_d.view(Lq, C), dev(t["o_w"], True), dev(t["o_b"]), hid_f, out=h1_b)   # operand of the next projection
    kv2_d = df.linear(dev(t["text"][0], True), dev(t["kv2_w"], True))    # [77, 2C]: C key columns, C value columns
    kvp = df.pack_text_kv(kv2_d, 1, TL, 1, C)
    w2, s2, t2 = fold(t["q2_w"], t["ln2_g"], t["ln2_b"])
    a2p = df.cross_attn_packed(df.pack_rows(h1_b), w2, s2, t2, kvp, 1, Lq, C, TL, 1, 0)
    a2_d = unpack_rows(host(a2p), Lq, C)[0]
    check(a2_d, a2, True, "cfg2 cross-attention output", say=say)
    out = df.linear_packed(a2p, df.pack_linear_weight(dev(t["o2_w"], True)), Lq, C, C, bias=dev(t["o2_b"]),
                           residual=h1_d, want=("f32",))["f32"]
    check(host(out), ref, True, "cfg2 layer output", say=say)
    # the stale rows matter: with the stale buffers replaced by the patch-free projection the result moves
    far = rel_l2(ops.attn_displaced(qkv[None, :, :C], qkv[None, :, C:2 * C], qkv[None, :, 2 * C:],
                                    np.zeros_like(k_stale), np.zeros_like(v_stale), heads, patch, N)[0], a1)
    say("   oracle: self-attention with zeroed stale rows is", far, "away")
    assert far > 5 * TOL_BF16


def test_config3_groupnorm_conv_silu_chain():
    """Configuration 3 as a chain: corrected GroupNorm of the 32-row patch (stale sums of the other three patches),
    then the 3x3 convolution with the stale halo rows and SiLU.  The convolution's stale input is what the previous
    step left: the GroupNorm of the stale full image."""
    t = configs.conv_gn_stage()
    m = t["meta"]
    H, C, N, G = m["H"], m["C"], m["N"], m["G"]
    R = H // N
    say("cfg3 chain", m)
    xs = t["x_stale"]
    st = ops.patch_group_sums(xs, G, N).astype(np.float32)
    gn_stale, _ = ops.groupnorm_stale(xs, ops.group_sums(xs, G)[None], t["gamma"], t["beta"], G, 0, 1, m["eps"])
    gn_stale = round_bf16(gn_stale.astype(np.float32))                    # the stored conv input is bf16
    for i in (0, 2):
        xf = t["x_full"][:, i * R:(i + 1) * R]
        r1, _ = ops.groupnorm_stale(xf, st, t["gamma"], t["beta"], G, i, N, m["eps"])
        r2 = ops.conv3x3_halo(r1, gn_stale, t["conv_w"], t["conv_b"], i, N, 1, 1)
        g1, _ = df.groupnorm_stale(dev(xf, True), dev(st), dev(t["gamma"]), dev(t["beta"]), G, i, N, m["eps"])
        g2 = df.conv3x3_halo(g1, dev(gn_stale, True), dev(t["conv_w"], True), dev(t["conv_b"]), i, N, 1, 1)
        check(host(g1), r1, True, "cfg3 chain patch %d GroupNorm" % i, say=say)
        check(host(g2), r2, True, "cfg3 chain patch %d conv+SiLU" % i, say=say)


# ---------------------------------------------------------------------------------------------------------------
# layer shapes of the 3840x3840 share (480x480 latent, N=8: 60 latent rows per patch)
# ---------------------------------------------------------------------------------------------------------------

def test_share_3840_layer_shapes():
    """One GroupNorm, one convolution (level 0: 60 x 480 pixels, 320 channels) and one self-attention (level 2:
    1800 queries against 14400 keys, 20 heads) at the shapes of one of 8 row patches of a 3840x3840 image."""
    N, patch = 8, 3
    # GroupNorm + convolution at level 0
    H, W, C, G = 480, 480, 320, 32
    R = H // N
    x = round_bf16(normal(61, "x", (1, R + 2, W, C)))                     # the patch's rows and the two halo rows
    w = round_bf16(normal(61, "w", (C, 3, 3, C), std=1.0 / math.sqrt(9 * C)))
    b = normal(61, "b", (C,), std=0.1)
    gamma, beta = normal(61, "g", (C,), std=0.1, mean=1.0), normal(61, "be", (C,), std=0.1)
    st = (np.abs(normal(61, "st", (N, 1, G, 2))) * np.array([100.0, R * W * C / G])).astype(np.float32)
    st[..., 1] += st[..., 0] ** 2 / (R * W * C / G)                       # sums of squares consistent with the sums
    xf = x[:, 1:R + 1]
    ref, _ = ops.groupnorm_stale(xf, st, gamma, beta, G, patch, N, 1e-5, 0, True)
    y, _ = df.groupnorm_stale(dev(xf, True), dev(st), dev(gamma), dev(beta), G, patch, N, 1e-5, 0, True)
    check(host(y), ref, True, "3840 share GroupNorm 60x480x320", say=say)
    # the same 60 x 480 patch as the middle one of three (a 180-row image): the kernel's work is that of the share,
    # the oracle's full-image convolution stays at seconds; stale rows other than s-1 and e cannot reach the output
    Nc, pc = 3, 1
    stale = normal(61, "stale", (1, Nc * R, W, C))
    stale[:, pc * R - 1] = x[:, 0]
    stale[:, (pc + 1) * R] = x[:, R + 1]
    stale = round_bf16(stale)
    ref = ops.conv3x3_halo(xf, stale, w, b, pc, Nc, 1, 0)
    yc = df.conv3x3_halo(dev(xf, True), dev(stale, True), dev(w, True), dev(b), pc, Nc, 1, 0)
    check(host(yc), ref, True, "3840 share conv 60x480 320->320", say=say)
    # self-attention at level 2
    t = _attn_case(62, 1, 14400, 1280, N, patch, True, stale_std=0.5)
    ref = ops.attn_displaced(t["q"], t["kf"], t["vf"], t["ks"], t["vs"], 20, patch, N)
    o = df.attn_displaced(dev(t["q"], True), dev(t["kf"], True), dev(t["vf"], True), dev(t["ks"], True),
                          dev(t["vs"], True), 20, patch, N)
    check(host(o), ref, True, "3840 share attention 1800 x 14400 x 1280", say=say)


# ---------------------------------------------------------------------------------------------------------------
# vertical strips (Section 5.1, Baselines: the patch split may run along either direction)
# ---------------------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_buffer_refresh_columns_bit_exact(dtype):
    g = torch.Generator().manual_seed(6)
    B, H, W, C, N = 2, 5, 12, 24, 4
    full = torch.randn(B, H, W, C, generator=g).to(dtype).to(DEV)
    Wp = W // N
    bits = torch.int16 if dtype == torch.bfloat16 else torch.int32
    for i in range(N):
        patch = torch.randn(B, H, Wp, C, generator=g).to(dtype).to(DEV)
        want = full.clone()
        want[:, :, i * Wp:(i + 1) * Wp] = patch
        got = df.buffer_refresh_cols(full.clone(), patch, i, N)
        torch.cuda.synchronize()
        assert torch.equal(got.view(bits), want.view(bits))


@pytest.mark.parametrize("B,H,W,Cin,Cout,N,stride,bf16", [
    (1, 16, 16, 32, 32, 2, 1, False),    # the tiny configuration, split along columns
    (2, 6, 12, 5, 7, 3, 1, False),       # odd channel counts
    (1, 8, 16, 8, 12, 4, 2, False),      # stride 2: only the left column is needed
    (1, 8, 8, 4, 64, 2, 1, True),        # 4 input channels
    (1, 8, 8, 128, 4, 2, 1, True),       # 4 output channels
    (2, 12, 16, 64, 96, 4, 1, True),     # MFMA tile path, ragged M and N tiles
    (1, 24, 16, 96, 64, 4, 2, True),     # MFMA, stride 2
    (1, 40, 32, 64, 320, 2, 1, True),    # MFMA, several N tiles
    (1, 128, 128, 320, 320, 4, 1, True), # configuration 3's layer, vertical strips of 32 columns
])
def test_conv_halo_columns_all_patches(B, H, W, Cin, Cout, N, stride, bf16):
    say("conv columns", B, H, W, Cin, Cout, N, stride, bf16)
    full, stale, w, b = _conv_case(12, B, H, W, Cin, Cout, bf16)
    Wp = W // N
    for i in (range(N) if H * W <= 4096 else (0, 1, N - 1)):
        xf = np.ascontiguousarray(full[:, :, i * Wp:(i + 1) * Wp])
        ref = ops.conv3x3_halo(xf, stale, w, b, i, N, stride, 1, split_axis=2)
        y = df.conv3x3_halo_cols(dev(xf, bf16), dev(stale, bf16), dev(w, bf16), dev(b), i, N, stride, 1)
        check(host(y), ref, bf16, "conv columns patch %d" % i, say=say)
    # the columns next to the strip matter and nothing else of the stale buffer does
    i = N - 1 if N > 1 else 0
    xf = np.ascontiguousarray(full[:, :, i * Wp:(i + 1) * Wp])
    far = stale.copy()
    far[:, :, :max(i * Wp - 1, 0)] = 77.0
    far[:, :, i * Wp:(i + 1) * Wp] = -77.0
    y0 = df.conv3x3_halo_cols(dev(xf, bf16), dev(stale, bf16), dev(w, bf16), dev(b), i, N, stride, 0)
    y1 = df.conv3x3_halo_cols(dev(xf, bf16), dev(far, bf16), dev(w, bf16), dev(b), i, N, stride, 0)
    np.testing.assert_array_equal(host(y0), host(y1))


@pytest.mark.parametrize("B,H,W,C,heads,N,patch,bf16", [
    (1, 16, 16, 32, 1, 2, 0, False),     # the tiny configuration's token grid
    (2, 6, 9, 128, 2, 3, 1, False),      # d = 64 in float32
    (1, 16, 32, 128, 2, 4, 2, True),     # bf16 MFMA kernel: 8 own tokens of every 32
    (2, 10, 60, 64, 1, 4, 3, True),      # ragged tiles, batch 2
    (1, 40, 60, 192, 3, 4, 1, True),     # level-2 grid of the 1280x1920 image as four vertical strips, split keys
])
def test_attention_displaced_columns(B, H, W, C, heads, N, patch, bf16):
    say("attn columns", B, H, W, C, heads, N, patch, bf16)
    L, Wp = H * W, W // N
    rnd = round_bf16 if bf16 else (lambda a: a)
    kfull, vfull = normal(23, "k", (B, L, C)), normal(23, "v", (B, L, C))
    own = np.array([r * W + c for r in range(H) for c in range(patch * Wp, (patch + 1) * Wp)])
    q = rnd(normal(23, "q", (B, len(own), C)))
    kf, vf = rnd(kfull[:, own].copy()), rnd(vfull[:, own].copy())
    ks = rnd(kfull + normal(23, "kn", (B, L, C), std=0.5))
    vs = rnd(vfull + normal(23, "vn", (B, L, C), std=0.5))
    ref = ops.attn_displaced(q, kf, vf, ks, vs, heads, patch, N, split_axis=2, hw=(H, W))
    o = df.attn_displaced_cols(dev(q, bf16), dev(kf, bf16), dev(vf, bf16), dev(ks, bf16), dev(vs, bf16), heads, H, W,
                               patch, N)
    check(host(o), ref, bf16, "attn columns", say=say)
    ks2, vs2 = ks.copy(), vs.copy()
    ks2[:, own], vs2[:, own] = 50.0, -50.0                  # the strip's own tokens of the stale buffers are not read
    o2 = df.attn_displaced_cols(dev(q, bf16), dev(kf, bf16), dev(vf, bf16), dev(ks2, bf16), dev(vs2, bf16), heads, H, W,
                                patch, N)
    np.testing.assert_array_equal(host(o2), host(o))
    # and the splice matters: as horizontal strips the same buffers give something else
    far = rel_l2(ops.attn_displaced(q, kf, vf, ks, vs, heads, patch, N), ref)
    assert far > (5 * TOL_BF16 if bf16 else 1e-3)


def test_tiny_block_chain_columns_f32():
    """The tiny configuration's GroupNorm -> conv3x3 -> attention block on vertical strips."""
    t = configs.tiny_block()
    m = t["meta"]
    H, W, C, N, G = m["H"], m["W"], m["C"], m["N"], m["G"]
    x, xs = t["x_full"], t["x_full"] + t["stale_noise"]
    gn_s, _ = ops.groupnorm_stale(xs, ops.group_sums(xs, G)[None], t["gamma"], t["beta"], G, 0, 1, m["eps"])
    st_stats = ops.patch_group_sums(xs, G, N, axis=2).astype(np.float32)
    conv_s = ops.conv3x3_full(gn_s, t["conv_w"], t["conv_b"])
    kv_s = conv_s.reshape(1, H * W, C)
    Wp = W // N
    for i in range(N):
        xf = np.ascontiguousarray(x[:, :, i * Wp:(i + 1) * Wp])
        r1, _ = ops.groupnorm_stale(xf, st_stats, t["gamma"], t["beta"], G, i, N, m["eps"])
        r2 = ops.conv3x3_halo(r1, gn_s, t["conv_w"], t["conv_b"], i, N, split_axis=2)
        tok = r2.reshape(1, H * Wp, C)
        r3 = ops.attn_displaced(tok, tok, tok, kv_s, kv_s, 1, i, N, split_axis=2, hw=(H, W))
        g1, _ = df.groupnorm_stale(dev(xf), dev(st_stats), dev(t["gamma"]), dev(t["beta"]), G, i, N, m["eps"])
        g2 = df.conv3x3_halo_cols(g1, dev(gn_s), dev(t["conv_w"]), dev(t["conv_b"]), i, N)
        gt = g2.reshape(1, H * Wp, C)
        g3 = df.attn_displaced_cols(gt, gt, gt, dev(kv_s), dev(kv_s), 1, H, W, i, N)
        for nm, g, r in (("gn", g1, r1), ("conv", g2, r2), ("attn", g3, r3)):
            check(host(g), r.reshape(host(g).shape), False, "tiny block columns patch %d %s" % (i, nm), say=say)


# ---------------------------------------------------------------------------------------------------------------
# Degenerate shapes: one-row patches (both halo rows come from the stale buffer, every output row is a boundary row),
# a one-pixel-wide image, one query row, one channel per group, one pixel per patch; and sizes that are no sizes.
# ---------------------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("bf16", [False, True])
def test_degenerate_one_row_patches_and_unit_widths(bf16):
    say("degenerate", bf16)
    # convolution: H = N (patches of one row), then W = 1
    for (B, H, W, Cin, Cout, N) in ((1, 4, 6, 64 if bf16 else 5, 64 if bf16 else 3, 4), (2, 6, 1, 8, 8, 3)):
        full, stale, w, b = _conv_case(71, B, H, W, Cin, Cout, bf16)
        R = H // N
        for i in range(N):
            xf = full[:, i * R:(i + 1) * R]
            ref = ops.conv3x3_halo(xf, stale, w, b, i, N, 1, 0)
            y = df.conv3x3_halo(dev(xf, bf16), dev(stale, bf16), dev(w, bf16), dev(b), i, N, 1, 0)
            check(host(y), ref, bf16, "conv %d-row patch %d (W=%d)" % (R, i, W), say=say)
    # attention: one query row per patch (Lq = 1), d = 64
    t = _attn_case(72, 1, 8, 64, 8, 3, bf16)
    ref = ops.attn_displaced(t["q"], t["kf"], t["vf"], t["ks"], t["vs"], 1, 3, 8)
    o = df.attn_displaced(dev(t["q"], bf16), dev(t["kf"], bf16), dev(t["vf"], bf16), dev(t["ks"], bf16), dev(t["vs"], bf16), 1, 3, 8)
    check(host(o), ref, bf16, "attention with one query", say=say)
    # GroupNorm: one channel per group, one pixel per patch (its variance comes from the other patches' sums alone)
    for (B, H, W, C, G, N, patch) in ((1, 4, 1, 8, 8, 4, 2), (2, 2, 3, 16, 16, 2, 0)):
        full, st, gamma, beta = _gn_case(73, B, H, W, C, G, N, bf16)
        R = H // N
        xf = full[:, patch * R:(patch + 1) * R]
        ref, ref_fs = ops.groupnorm_stale(xf, st, gamma, beta, G, patch, N, 1e-5, 0, False)
        y, fs = df.groupnorm_stale(dev(xf, bf16), dev(st), dev(gamma), dev(beta), G, patch, N, 1e-5, 0, False)
        check(host(y), ref, bf16, "gn one channel per group, %d pixels" % (R * W), say=say)
        assert rel_l2(host(fs), ref_fs) < 1e-5


def test_empty_and_invalid_sizes_are_errors_not_launches():
    z = lambda *s: torch.zeros(*s, device=DEV)
    w3 = z(4, 3, 3, 4)
    with pytest.raises(df.DfError):
        df.conv3x3_halo(z(0, 2, 2, 4), z(0, 4, 2, 4), w3, z(4), 0, 2, 1, 0)              # empty batch
    with pytest.raises(df.DfError):
        df.conv3x3_halo(z(1, 2, 2, 4), z(1, 4, 2, 4), w3, z(4), 2, 2, 1, 0)              # patch index == N
    with pytest.raises(df.DfError):
        df.conv3x3_halo(z(1, 2, 2, 4), z(1, 4, 2, 4), w3, z(4), 0, 2, 3, 0)              # stride 3
    with pytest.raises(df.DfError):
        df.conv3x3_halo(z(1, 2, 2, 4), None, w3, z(4), 0, 2, 1, 0)                       # stale buffer missing with N > 1
    with pytest.raises(df.DfError):
        df.attn_displaced(z(1, 0, 64), z(1, 0, 64), z(1, 0, 64), z(1, 8, 64), z(1, 8, 64), 1, 0, 2)   # no queries
    with pytest.raises(df.DfError):
        df.attn_displaced(z(1, 4, 64), z(1, 4, 64), z(1, 4, 64), z(1, 8, 64), z(1, 8, 64), 1, 0, 2, scale=0.0)
    with pytest.raises(df.DfError):
        df.groupnorm_stale(z(1, 0, 2, 8), z(2, 1, 4, 2), torch.ones(8, device=DEV), z(8), 4, 0, 2)    # no rows
    with pytest.raises(df.DfError):
        df.linear(z(0, 64).to(torch.bfloat16), z(32, 64).to(torch.bfloat16), z(32))       # no rows
    with pytest.raises(df.DfError):
        df.buffer_refresh(z(1, 8, 4), z(1, 0, 4), 0, 4)                                   # fresh block of the wrong size
