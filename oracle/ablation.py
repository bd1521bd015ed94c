"""Test infrastructure (CPU oracle only; never imported by the product path).

Numerical re-run of the paper's two ablations on synthetic data (Section 5.3, GroupNorm; Section 4 / Section 5.3,
warm-up steps): the full multi-device method is emulated with the float64 oracle - every one of the N patches runs a
DISPLACED step against the state left by the previous step, then the refreshed rows of all patches are merged (the
AllGather) - for each GroupNorm statistic mode and several warm-up counts, and the final latent is compared with the
one produced by synchronous (FULL) steps throughout.

    python -m oracle.ablation [--steps 8] [--H 32 --W 16 --N 4]
"""
import argparse
import math

import numpy as np

from df_inputs import configs, unet_table as ut
from oracle import ops, unet as ounet


def _merge_patch_rows(dst, src, name, i, N):
    """Copies patch i's slots of stale entry `name` from src to dst (what the AllGather delivers)."""
    a, b = dst[name], src[name]
    if name.endswith(".stats"):          # [N, B, G, 2]
        a[i] = b[i]
    else:                                # [B, rows or tokens, ...]: the patch owns a contiguous 1/N of axis 1
        n = a.shape[1] // N
        a[:, i * n:(i + 1) * n] = b[:, i * n:(i + 1) * n]


def run(cfg, weights, t, sigmas, n_warmup, stat_mode):
    """Latent after the Euler loop with `n_warmup` synchronous steps, then displaced steps on all N patches."""
    bl = ut.blocks(cfg)
    P = ounet.Params(weights)
    N, R = cfg.N, cfg.H // cfg.N
    x = t["x_prev"].astype(np.float64) * sigmas[0]
    stale = {}
    for k in range(len(sigmas) - 1):
        sc = 1.0 / math.sqrt(sigmas[k] ** 2 + 1)
        if k < n_warmup:
            eps = ounet.unet_step(cfg, bl, P, x * sc, t["emb"], t["text"], stale, mode=ounet.FULL)
        else:
            eps = np.empty_like(x)
            new = {kk: v.copy() for kk, v in stale.items()}
            for i in range(N):
                mine = {kk: v.copy() for kk, v in stale.items()}
                rows = slice(i * R, (i + 1) * R)
                eps[:, rows] = ounet.unet_step(cfg, bl, P, x[:, rows] * sc, t["emb"], t["text"], mine, i,
                                               ounet.DISPLACED, stat_mode=stat_mode)
                for name in new:
                    _merge_patch_rows(new, mine, name, i, N)
            stale = new
        x = ounet.euler_update(x, eps, sigmas[k], sigmas[k + 1])
    return x


def table(H=32, W=16, N=4, steps=8, seed=21, warmups=(1, 2, 4)):
    cfg = ut.UNetCfg(H=H, W=W, N=N, **ut.SMALL)
    weights = configs.unet_weights(cfg, seed=seed, threads=8)
    t = configs.unet_inputs(cfg, seed=seed)
    sig = list(np.geomspace(8.0, 0.05, steps + 1))
    ref = run(cfg, weights, t, sig, steps, ops.STAT_SUMS)          # synchronous throughout
    names = {ops.STAT_SUMS: "sums (exact statistics of the scatter output)", ops.STAT_EQ2: "Eq. 2 as printed",
             ops.STAT_SEPARATE: "separate GN", ops.STAT_STALE: "stale GN"}
    out = []
    for mode, label in names.items():
        row = []
        for nw in warmups:
            x = run(cfg, weights, t, sig, nw, mode)
            row.append(float(np.linalg.norm(x - ref) / np.linalg.norm(ref)))
        out.append((label, row))
    return warmups, out


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--H", type=int, default=32)
    ap.add_argument("--W", type=int, default=16)
    ap.add_argument("--N", type=int, default=4)
    a = ap.parse_args()
    warmups, rows = table(a.H, a.W, a.N, a.steps)
    print("relative L2 distance of the final latent to the synchronous run; columns: warm-up steps", list(warmups))
    for label, row in rows:
        print(f"{label:50s}", "  ".join(f"{v:.4f}" for v in row))
