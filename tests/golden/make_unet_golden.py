#!/usr/bin/env python3
"""Writes the oracle's expected outputs for the full-size UNet configurations.

Calls only df_inputs (seeded inputs) and oracle/ (float64 CPU reference).  The GPU tests load the
.npz files it writes and compare the HIP path against them, because the full-image oracle pass
takes minutes of CPU time.

  python tests/golden/make_unet_golden.py cfg4     # 160x240 latent, N=8, patch 3 (SDXL-shaped)
  python tests/golden/make_unet_golden.py cfg4far  # same, but the current input is 0.5 N(0,1) away from the previous one
  python tests/golden/make_unet_golden.py loop     # 6-step Euler loop at a 64x64 latent
  python tests/golden/make_unet_golden.py cfg5 [checkpoint_dir]   # 10-step Euler loop at the 256x256 latent, N=4
                                                   # (about two hours; resumes from the checkpoint directory)

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
    # the same FULL step, but the patch's current input differs from the previous step's by 0.5 N(0,1): the
    # DISPLACED result is then far (many tolerances) from the previous step's rows, so a step that confused
    # fresh and stale data cannot pass
    "cfg4far": dict(H=160, W=240, N=8, patch=3, seed=4, arch="SDXL", stale_std=0.5),
    # multi-step loop of configuration 5 at a latent size the oracle finishes in minutes: SDXL architecture,
    # 64x64 latent, N=4 (16 latent rows per patch), patch 1, 6 Euler steps (1 FULL + 5 DISPLACED with refresh)
    "loop": dict(H=64, W=64, N=4, patch=1, seed=5, arch="SDXL", steps=6),
    # the multi-step configuration at its stated size: 2048x2048 image = 256x256 latent, N=4 (64 latent rows),
    # patch 1, 10 Euler steps (1 FULL + 9 DISPLACED with refresh)
    "cfg5": dict(H=256, W=256, N=4, patch=1, seed=5, arch="SDXL", steps=10),
}

# sigma ladder of the multi-step loop: geometric from 14.6 to 0.03 (the range of SDXL's Euler schedule)
def sigma_ladder(steps):
    return [14.6 * (0.03 / 14.6) ** (k / steps) for k in range(steps + 1)]


def _save_state(ckpt, k, stale, eps_list, x_list, x):
    """Checkpoint of the loop after step k (a step of the full-size loop takes many minutes of CPU time): the stale
    state as one .npy per buffer, the results so far, and a marker written last."""
    os.makedirs(ckpt, exist_ok=True)
    marker = os.path.join(ckpt, "done_step.txt")
    if os.path.exists(marker):
        os.remove(marker)
    names = sorted(stale)
    for j, nm in enumerate(names):
        np.save(os.path.join(ckpt, "stale_%04d.npy" % j), stale[nm])
    np.savez(os.path.join(ckpt, "results.npz"), eps=np.stack(eps_list), xs=np.stack(x_list), x=x)
    with open(os.path.join(ckpt, "names.txt"), "w") as f:
        f.write("\n".join(names))
    with open(marker, "w") as f:
        f.write(str(k))


def _load_state(ckpt):
    marker = os.path.join(ckpt, "done_step.txt")
    if not os.path.exists(marker):
        return None
    k = int(open(marker).read())
    names = open(os.path.join(ckpt, "names.txt")).read().split("\n")
    stale = {nm: np.load(os.path.join(ckpt, "stale_%04d.npy" % j)) for j, nm in enumerate(names)}
    r = np.load(os.path.join(ckpt, "results.npz"))
    return k, stale, list(r["eps"]), list(r["xs"]), r["x"]


def main_loop(which, ckpt=None):
    """Euler loop (Section 3, Eq. 1): x <- x + (sigma_{k+1} - sigma_k) * eps on the patch's latent rows; step 0
    computes the full image and fills the stale state, later steps compute the patch only and refresh its rows.
    With a checkpoint directory the state is saved after every step and an interrupted run resumes from it."""
    r = RECIPES[which]
    cfg = ut.UNetCfg(H=r["H"], W=r["W"], N=r["N"], **getattr(ut, r["arch"]))
    weights = configs.unet_weights(cfg, seed=r["seed"], threads=8)
    t = configs.unet_inputs(cfg, seed=r["seed"])
    bl = ut.blocks(cfg)
    P = ounet.Params(weights)
    sig = sigma_ladder(r["steps"])
    R = cfg.H // cfg.N
    i = r["patch"]
    state = _load_state(ckpt) if ckpt else None
    if state is None:
        stale = {}
        x_full = t["x_prev"].astype(np.float64) * sig[0]                      # noisy latent at sigma_0
        t0 = time.time()
        eps = ounet.unet_step(cfg, bl, P, x_full / np.sqrt(sig[0] ** 2 + 1), t["emb"], t["text"], stale, mode=ounet.FULL)
        print("step 0 FULL", round(time.time() - t0, 1), "s", flush=True)
        x = ounet.euler_update(x_full, eps, sig[0], sig[1])[:, i * R:(i + 1) * R]
        eps_list = [eps[:, i * R:(i + 1) * R]]
        x_list = [x]
        done = 0
        if ckpt:
            _save_state(ckpt, 0, stale, eps_list, x_list, x)
    else:
        done, stale, eps_list, x_list, x = state
        print("resuming after step", done, flush=True)
    for k in range(done + 1, r["steps"]):
        t0 = time.time()
        e = ounet.unet_step(cfg, bl, P, x / np.sqrt(sig[k] ** 2 + 1), t["emb"], t["text"], stale, i, ounet.DISPLACED)
        x = ounet.euler_update(x, e, sig[k], sig[k + 1])
        eps_list.append(e)
        x_list.append(x)
        print("step", k, "DISPLACED", round(time.time() - t0, 1), "s", flush=True)
        if ckpt:
            _save_state(ckpt, k, stale, eps_list, x_list, x)
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"unet_{which}_eps.npz")
    np.savez_compressed(out, eps=np.stack(eps_list).astype(np.float32), x=np.stack(x_list).astype(np.float32),
                        sigmas=np.array(sig), H=r["H"], W=r["W"], N=r["N"], patch=i, seed=r["seed"], steps=r["steps"])
    print("wrote", out, os.path.getsize(out), "bytes")



def main(which):
    r = RECIPES[which]
    cfg = ut.UNetCfg(H=r["H"], W=r["W"], N=r["N"], **getattr(ut, r["arch"]))
    t0 = time.time()
    weights = configs.unet_weights(cfg, seed=r["seed"], threads=8)
    print("weights", round(time.time() - t0, 1), "s", flush=True)
    t = configs.unet_inputs(cfg, seed=r["seed"], stale_std=r.get("stale_std", 0.02))
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
    which = sys.argv[1] if len(sys.argv) > 1 else "cfg4"
    if "steps" in RECIPES[which]:
        main_loop(which, sys.argv[2] if len(sys.argv) > 2 else None)      # optional checkpoint directory
    else:
        main(which)
