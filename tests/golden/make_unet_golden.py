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
    # the same loop on the reduced-width network (seconds): self-check of the checkpoint / resume logic
    "smallloop": dict(H=32, W=16, N=4, patch=1, seed=5, arch="SMALL", steps=4),
}

# sigma ladder of the multi-step loop: geometric from 14.6 to 0.03 (the range of SDXL's Euler schedule)
def sigma_ladder(steps):
    return [14.6 * (0.03 / 14.6) ** (k / steps) for k in range(steps + 1)]


class _Checkpoint:
    """Progress of the loop on disk, block by block (a step of the full-size loop takes many minutes of CPU time and
    the machine may stop the run at any point): every stale buffer as one .npy, the activation and the pending skip
    connections after the last finished block, the results of the finished steps, and a marker written last.  Files
    are replaced atomically, and re-running a block is harmless (a FULL step only writes the buffers; a DISPLACED
    step never reads the rows it refreshes), so a run killed at any point resumes correctly."""

    def __init__(self, path, blocks):
        self.path, self.blocks = path, blocks
        os.makedirs(path, exist_ok=True)
        self.index = {}                                   # stale name -> file number
        idx = os.path.join(path, "names.txt")
        if os.path.exists(idx):
            for j, nm in enumerate(open(idx).read().split("\n")):
                if nm:
                    self.index[nm] = j

    def _put(self, name, arr):
        tmp = os.path.join(self.path, name + ".tmp.npy")
        np.save(tmp, arr)
        os.replace(tmp, os.path.join(self.path, name + ".npy"))

    def _mark(self, text):
        tmp = os.path.join(self.path, "progress.tmp")
        with open(tmp, "w") as f:
            f.write(text)
        os.replace(tmp, os.path.join(self.path, "progress.txt"))

    def block_done(self, step, n, h, skips, stale, saved_skips):
        """After the n-th entry of the block list of step `step`."""
        name = self.blocks[n - 1][1] if len(self.blocks[n - 1]) > 1 else ""
        if name:
            for nm in stale:
                if nm.startswith(name + "."):
                    if nm not in self.index:
                        self.index[nm] = len(self.index)
                        with open(os.path.join(self.path, "names.txt"), "a") as f:
                            f.write(nm + "\n")
                    self._put("stale_%04d" % self.index[nm], stale[nm])
        for j in range(saved_skips[0], len(skips)):
            self._put("skip_%02d" % j, skips[j])
        saved_skips[0] = len(skips)
        self._put("h", h)
        self._mark("%d %d %d" % (step, n, len(skips)))

    def step_done(self, step, eps_list, x_list, x):
        tmp = os.path.join(self.path, "results.tmp.npz")
        np.savez(tmp, eps=np.stack(eps_list), xs=np.stack(x_list), x=x)
        os.replace(tmp, os.path.join(self.path, "results.npz"))
        self._mark("%d %d %d" % (step + 1, 0, 0))

    def load(self):
        """(step in progress, blocks done in it, resume tuple or None, stale, eps_list, x_list, x) or None."""
        mark = os.path.join(self.path, "progress.txt")
        if not os.path.exists(mark):
            return None
        step, n, nsk = (int(v) for v in open(mark).read().split())
        stale = {nm: np.load(os.path.join(self.path, "stale_%04d.npy" % j)) for nm, j in self.index.items()
                 if os.path.exists(os.path.join(self.path, "stale_%04d.npy" % j))}
        eps_list, x_list, x = [], [], None
        res = os.path.join(self.path, "results.npz")
        if os.path.exists(res):
            r = np.load(res)
            eps_list, x_list, x = list(r["eps"]), list(r["xs"]), r["x"]
        resume = None
        if n > 0:
            skips = [np.load(os.path.join(self.path, "skip_%02d.npy" % j)) for j in range(nsk)]
            resume = (n, np.load(os.path.join(self.path, "h.npy")), skips)
        return step, n, resume, stale, eps_list, x_list, x


def main_loop(which, ckpt=None, out_dir=None):
    """Euler loop (Section 3, Eq. 1): x <- x + (sigma_{k+1} - sigma_k) * eps on the patch's latent rows; step 0
    computes the full image and fills the stale state, later steps compute the patch only and refresh its rows.
    With a checkpoint directory the progress is saved after every block and an interrupted run resumes from it."""
    r = RECIPES[which]
    cfg = ut.UNetCfg(H=r["H"], W=r["W"], N=r["N"], **getattr(ut, r["arch"]))
    weights = configs.unet_weights(cfg, seed=r["seed"], threads=8)
    t = configs.unet_inputs(cfg, seed=r["seed"])
    bl = ut.blocks(cfg)
    P = ounet.Params(weights)
    sig = sigma_ladder(r["steps"])
    R = cfg.H // cfg.N
    i = r["patch"]
    ck = _Checkpoint(ckpt, bl) if ckpt else None
    state = ck.load() if ck else None
    step0, resume, stale, eps_list, x_list, x = 0, None, {}, [], [], None
    if state is not None:
        step0, n_done, resume, stale, eps_list, x_list, x = state
        print("resuming at step", step0, "after block", n_done, flush=True)
    for k in range(step0, r["steps"]):
        t0 = time.time()
        saved_skips = [len(resume[2]) if resume else 0]
        hook = (lambda n, h, skips, k=k: ck.block_done(k, n, h, skips, stale, saved_skips)) if ck else None
        if k == 0:
            x_full = t["x_prev"].astype(np.float64) * sig[0]                  # noisy latent at sigma_0
            eps = ounet.unet_step(cfg, bl, P, x_full / np.sqrt(sig[0] ** 2 + 1), t["emb"], t["text"], stale,
                                  mode=ounet.FULL, resume=resume, on_block=hook)
            x = ounet.euler_update(x_full, eps, sig[0], sig[1])[:, i * R:(i + 1) * R]
            e = eps[:, i * R:(i + 1) * R]
        else:
            e = ounet.unet_step(cfg, bl, P, x / np.sqrt(sig[k] ** 2 + 1), t["emb"], t["text"], stale, i,
                                ounet.DISPLACED, resume=resume, on_block=hook)
            x = ounet.euler_update(x, e, sig[k], sig[k + 1])
        resume = None
        eps_list.append(e)
        x_list.append(x)
        print("step", k, "FULL" if k == 0 else "DISPLACED", round(time.time() - t0, 1), "s", flush=True)
        if ck:
            ck.step_done(k, eps_list, x_list, x)
    out = os.path.join(out_dir or os.path.dirname(os.path.abspath(__file__)), f"unet_{which}_eps.npz")
    np.savez_compressed(out, eps=np.stack(eps_list).astype(np.float32), x=np.stack(x_list).astype(np.float32),
                        sigmas=np.array(sig), H=r["H"], W=r["W"], N=r["N"], patch=i, seed=r["seed"], steps=r["steps"])
    print("wrote", out, os.path.getsize(out), "bytes")
    return out



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
