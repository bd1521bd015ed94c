"""Pins of the oracle's whole-step chain: the paper's cost figure for the layer
table, and the invariants of Section 4 (the synchronous first step is the
ordinary forward; displaced computation is exact when the stale activations
equal the fresh ones; one patch with N=1 is the full image)."""
import numpy as np
import pytest

from df_inputs import configs, unet_table as ut
from oracle import ops, unet


def test_layer_table_matches_paper_mac_count():
    # Section 3: 6,763 GMACs per step for a 1024x1024 image (128x128 latent) at CFG batch 2
    cfg = ut.UNetCfg(H=128, W=128, N=1, **ut.SDXL)
    m = ut.count_macs(cfg)
    assert abs(2 * m["total"] / 1e9 - 6763) / 6763 < 1e-3
    # Table 1: total MACs do not depend on the number of devices except through attention's
    # fixed key/value length: per-patch cost times N equals the full cost
    for N in (2, 4, 8):
        mp = ut.count_macs(ut.UNetCfg(H=128, W=128, N=N, **ut.SDXL))
        for k in ("conv", "self_attn", "cross_attn"):
            assert mp[k] * N == m[k]
    assert 2.5e9 < ut.num_params(cfg) < 2.6e9


def test_layer_table_shapes():
    cfg = ut.UNetCfg(H=160, W=240, N=8, **ut.SDXL)
    bl = ut.blocks(cfg)
    kinds = [b[0] for b in bl]
    assert kinds.count("res") == 2 * 3 + 2 + 3 * 3
    assert kinds.count("push") == 9 and kinds.count("down") == 2 and kinds.count("up") == 2
    specs = ut.weight_specs(cfg)
    names = [s[0] for s in specs]
    assert len(set(names)) == len(names)
    n_conv = sum(1 for n, sh, _ in specs if len(sh) == 4)
    n_gn = sum(1 for n, _, _ in specs if (".gn" in n) and n.endswith(".g"))
    n_attn = sum(1 for n in names if n.endswith("attn1.qkv.w"))
    n_ln = sum(1 for n in names if ".ln" in n and n.endswith(".g"))
    assert (n_conv, n_gn, n_attn, n_ln) == (40, 46, 70, 210)
    cat = [b for b in bl if b[0] == "res" and b[5]]
    assert [b[2] for b in cat] == [2560, 2560, 1920, 1920, 1280, 960, 960, 640, 640]


def _small(N, H=16, W=8, seed=7):
    cfg = ut.UNetCfg(H=H, W=W, N=N, **ut.SMALL)
    w = configs.unet_weights(cfg, seed=seed, threads=4)
    t = configs.unet_inputs(cfg, seed=seed)
    return cfg, ut.blocks(cfg), unet.Params(w), t


def test_displaced_with_one_patch_is_the_full_forward():
    cfg, bl, P, t = _small(1)
    stale = {}
    full = unet.unet_step(cfg, bl, P, t["x"], t["emb"], t["text"], stale, mode=unet.FULL)
    assert full.shape == (1, 16, 8, 4) and np.isfinite(full).all() and full.std() > 1e-3
    # different stale content must not matter when the single patch covers everything
    junk = {k: v + 3.0 for k, v in stale.items()}
    disp = unet.unet_step(cfg, bl, P, t["x"], t["emb"], t["text"], junk, 0, unet.DISPLACED, refresh=False)
    np.testing.assert_allclose(disp, full, rtol=1e-9, atol=1e-10)


@pytest.mark.parametrize("N", [2, 4])
def test_displaced_is_exact_when_stale_equals_fresh_and_patches_tile(N):
    cfg, bl, P, t = _small(N, H=16 if N == 2 else 32)
    stale = {}
    tr_full = {}
    full = unet.unet_step(cfg, bl, P, t["x"], t["emb"], t["text"], stale, mode=unet.FULL, trace=tr_full)
    R = cfg.H // N
    tiles = []
    for i in range(N):
        snap = {k: v.copy() for k, v in stale.items()}
        out = unet.unet_step(cfg, bl, P, t["x"][:, i * R:(i + 1) * R], t["emb"], t["text"], snap, i, unet.DISPLACED)
        tiles.append(out)
        # refresh with identical data leaves the buffers unchanged
        for k in stale:
            np.testing.assert_allclose(snap[k], stale[k], rtol=1e-9, atol=1e-9)
    np.testing.assert_allclose(np.concatenate(tiles, axis=1), full, rtol=1e-8, atol=1e-9)
    # Eq. 2 statistics are exact as well in that case
    out = unet.unet_step(cfg, bl, P, t["x"][:, :R], t["emb"], t["text"], {k: v.copy() for k, v in stale.items()},
                         0, unet.DISPLACED, stat_mode=ops.STAT_EQ2)
    np.testing.assert_allclose(out, full[:, :R], rtol=1e-8, atol=1e-9)


def test_displaced_uses_stale_context_and_refresh_touches_own_rows_only():
    cfg, bl, P, t = _small(2)
    stale = {}
    unet.unet_step(cfg, bl, P, t["x_prev"], t["emb"], t["text"], stale, mode=unet.FULL)
    full_now = unet.unet_step(cfg, bl, P, t["x"], t["emb"], t["text"], {}, mode=unet.FULL)
    before = {k: v.copy() for k, v in stale.items()}
    out = unet.unet_step(cfg, bl, P, t["x"][:, 8:], t["emb"], t["text"], stale, 1, unet.DISPLACED)
    err = np.linalg.norm(out - full_now[:, 8:]) / np.linalg.norm(full_now[:, 8:])
    assert 0 < err < 0.2          # close to, but not equal to, the synchronous result
    changed = 0
    for k, v in stale.items():
        if k.endswith(".stats"):
            np.testing.assert_array_equal(v[0], before[k][0])
            changed += int(np.abs(v[1] - before[k][1]).max() > 0)
        else:
            half = v.shape[1] // 2
            np.testing.assert_array_equal(v[:, :half], before[k][:, :half])
            changed += int(np.abs(v[:, half:] - before[k][:, half:]).max() > 0)
    assert changed == len(stale)
    # keys: one buffer per conv input, two per self-attention, one per GroupNorm
    specs = ut.weight_specs(cfg)
    n_conv = sum(1 for _, sh, _ in specs if len(sh) == 4)
    n_attn = sum(1 for n, _, _ in specs if n.endswith("attn1.qkv.w"))
    n_gn = sum(1 for n, _, _ in specs if ".gn" in n and n.endswith(".g"))
    assert len(stale) == n_conv + 2 * n_attn + n_gn


def test_euler_update():
    x = np.array([1.0, 2.0])
    np.testing.assert_allclose(unet.euler_update(x, np.array([0.5, -1.0]), 2.0, 1.5), [0.75, 2.5])


def test_ablation_emulation_invariants():
    """oracle/ablation.py emulates all N devices with the oracle.  Warm-up on every step is the synchronous run itself;
    with stale == fresh state and unchanged input a displaced step of all patches reproduces the synchronous eps, so
    one displaced step after an Euler step of size zero changes nothing."""
    import numpy as np
    from df_inputs import configs, unet_table as ut
    from oracle import ablation, ops
    cfg = ut.UNetCfg(H=16, W=8, N=2, **ut.SMALL)
    weights = configs.unet_weights(cfg, seed=5, threads=4)
    t = configs.unet_inputs(cfg, seed=5)
    sig = [2.0, 1.0, 0.5]
    ref = ablation.run(cfg, weights, t, sig, 2, ops.STAT_SUMS)
    assert np.array_equal(ablation.run(cfg, weights, t, sig, 5, ops.STAT_EQ2), ref)
    # sigma ladder with a zero-size first step: the displaced second step sees exactly the state it was built from
    flat = [2.0, 2.0, 1.0]
    a = ablation.run(cfg, weights, t, flat, 2, ops.STAT_SUMS)
    for mode in (ops.STAT_SUMS, ops.STAT_EQ2, ops.STAT_STALE):
        b = ablation.run(cfg, weights, t, flat, 1, mode)
        assert np.linalg.norm(a - b) / np.linalg.norm(a) < 1e-9, mode


def test_golden_loop_script_resumes_bit_identically(tmp_path):
    """The script that writes the multi-step golden values checkpoints after every block and may be killed at any
    point: a run interrupted twice (inside the FULL step and inside a DISPLACED step) and resumed must write exactly
    what an uninterrupted run writes."""
    import importlib.util
    import os
    spec = importlib.util.spec_from_file_location(
        "make_unet_golden", os.path.join(os.path.dirname(__file__), "golden", "make_unet_golden.py"))
    mk = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mk)
    plain = tmp_path / "plain"
    plain.mkdir()
    ref = np.load(mk.main_loop("smallloop", None, str(plain)))

    class Stop(Exception):
        pass

    ck, out = tmp_path / "ck", tmp_path / "resumed"
    out.mkdir()
    orig = mk._Checkpoint.block_done
    for stop_after in (7, 25, None):                 # 7 blocks in: FULL step; 25 more: inside a DISPLACED step
        calls = [0]

        def hooked(self, *a, **k):
            orig(self, *a, **k)
            calls[0] += 1
            if stop_after is not None and calls[0] == stop_after:
                raise Stop()
        mk._Checkpoint.block_done = hooked
        try:
            path = mk.main_loop("smallloop", str(ck), str(out))
        except Stop:
            continue
        finally:
            mk._Checkpoint.block_done = orig
    got = np.load(path)
    np.testing.assert_array_equal(got["eps"], ref["eps"])
    np.testing.assert_array_equal(got["x"], ref["x"])


def test_unet_vertical_strips_invariants():
    """Vertical strips (split_axis=2) through the whole step: with the buffers a FULL pass leaves on the same input
    every strip's DISPLACED output equals its columns of the FULL output and the strips tile it; transposing the
    image (and every 3x3 kernel) maps the column split onto the row split."""
    cfg = ut.UNetCfg(H=8, W=16, N=2, **ut.SMALL)
    weights = configs.unet_weights(cfg, seed=21, threads=4)
    t = configs.unet_inputs(cfg, seed=21, stale_std=0.4)
    bl = ut.blocks(cfg)
    P = unet.Params(weights)
    stale = {}
    full = unet.unet_step(cfg, bl, P, t["x_prev"], t["emb"], t["text"], stale, mode=unet.FULL, split_axis=2)
    Wp = cfg.W // cfg.N
    tiles = [unet.unet_step(cfg, bl, P, t["x_prev"][:, :, j * Wp:(j + 1) * Wp], t["emb"], t["text"],
                             {k: v.copy() for k, v in stale.items()}, j, unet.DISPLACED, split_axis=2)
             for j in range(cfg.N)]
    np.testing.assert_allclose(np.concatenate(tiles, axis=2), full, rtol=1e-9, atol=1e-10)
    # a new input for strip 1 with the old state: compare with the row split of the transposed problem
    xs = t["x"][:, :, Wp:2 * Wp]
    cols = unet.unet_step(cfg, bl, P, xs, t["emb"], t["text"], {k: v.copy() for k, v in stale.items()}, 1,
                           unet.DISPLACED, split_axis=2)
    assert np.abs(cols - tiles[1]).max() > 1e-3                       # the new input matters
    cfg_t = ut.UNetCfg(H=cfg.W, W=cfg.H, N=cfg.N, **ut.SMALL)
    wt = [(n, (np.ascontiguousarray(np.swapaxes(a, 1, 2)) if a.ndim == 4 else a)) for n, a in weights]
    Pt = unet.Params(wt)
    stale_t = {}
    unet.unet_step(cfg_t, ut.blocks(cfg_t), Pt, np.swapaxes(t["x_prev"], 1, 2), t["emb"], t["text"], stale_t,
                    mode=unet.FULL)
    rows = unet.unet_step(cfg_t, ut.blocks(cfg_t), Pt, np.swapaxes(xs, 1, 2), t["emb"], t["text"], stale_t, 1,
                           unet.DISPLACED)
    np.testing.assert_allclose(np.swapaxes(rows, 1, 2), cols, rtol=1e-8, atol=1e-9)
