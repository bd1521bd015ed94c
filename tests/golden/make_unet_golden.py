#!/usr/bin/env python3
"""Writes the oracle's expected outputs for the full-size UNet configurations.

Calls only df_inputs (seeded inputs) and oracle/ (float64 CPU reference).  The GPU tests load the
.npz files it writes and compare the HIP path against them, because the full-image oracle pass
takes minutes of CPU time.

  python tests/golden/make_unet_golden.py cfg4     # 160x240 latent, N=8, patch 3 (SDXL-shaped)

Stored: eps of the FULL step on x_prev, eps of the DISPLACED step of the patch on x with the stale
state that FULL step left (both float32), and the recipe's parameters.
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from df_inputs import configs, unet_table as ut  # noqa: E402
from oracle import unet as ounet  # noqa: E402

RECIPES = {
    "cfg4": dict(H=160, W=240, N=8, patch=3, seed=4, arch="SDXL"),
}


def main(which):
    r = RECIPES[which]
    cfg = ut.UNetCfg(H=r["H"], W=r["W"], N=r["N"], **getattr(ut, r["arch"]))
    t0 = time.time()
    weights = configs.unet_weights(cfg, seed=r["seed"], threads=8)
    print("weights", round(time.time() - t0, 1), "s", flush=True)
    t = configs.unet_inputs(cfg, seed=r["seed"])
    bl = ut.blocks(cfg)
    P = ounet.Params(weights)
    stale = {}
    t0 = time.time()
    eps_full = ounet.unet_step(cfg, bl, P, t["x_prev"], t["emb"], t["text"], stale, mode=ounet.FULL)
    print("FULL", round(time.time() - t0, 1), "s", flush=True)
    R = cfg.H // cfg.N
    i = r["patch"]
    t0 = time.time()
    eps_disp = ounet.unet_step(cfg, bl, P, t["x"][:, i * R:(i + 1) * R], t["emb"], t["text"], stale, i, ounet.DISPLACED)
    print("DISPLACED", round(time.time() - t0, 1), "s", flush=True)
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"unet_{which}_eps.npz")
    np.savez_compressed(out, eps_full=eps_full.astype(np.float32), eps_disp=eps_disp.astype(np.float32),
                        H=r["H"], W=r["W"], N=r["N"], patch=i, seed=r["seed"])
    print("wrote", out, os.path.getsize(out), "bytes")


if __name__ == "__main__":
    main(sys.argv[1] if len(sys.argv) > 1 else "cfg4")
