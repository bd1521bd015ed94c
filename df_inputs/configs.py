"""Seeded raw tensors of the benchmark configurations.

Only draws of random numbers and rounding to the storage dtype happen here.
Tensors that the method derives from others (projected K/V, GroupNorm sums,
stale buffers left by a full-image pass) are built by whoever consumes these.

Stale-activation noise follows the input-similarity measurement of the paper
(Section 5.3, Input similarity: consecutive steps differ by 0.02 on average
over a [-4, 4] range): stale = fresh + sigma * N(0,1) with sigma 0.02 (0.05
in the tiny configuration).
"""
import math
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from .rng import normal, round_bf16, to_bf16_bits
from .unet_table import weight_specs


def tiny_block(seed=1, H=16, W=16, C=32, N=2):
    """Configuration 1: fp32 GroupNorm -> conv3x3 -> single-head attention block."""
    t = {}
    t["x_full"] = normal(seed, "x_full", (1, H, W, C))
    t["stale_noise"] = normal(seed, "stale_noise", (1, H, W, C), std=0.05)
    t["gamma"] = normal(seed, "gn.gamma", (C,), std=0.1, mean=1.0)
    t["beta"] = normal(seed, "gn.beta", (C,), std=0.1)
    t["conv_w"] = normal(seed, "conv.w", (C, 3, 3, C), std=1.0 / math.sqrt(9 * C))
    t["conv_b"] = normal(seed, "conv.b", (C,), std=0.02)
    for nm in ("wq", "wk", "wv", "wo"):
        t[nm] = normal(seed, "attn." + nm, (C, C), std=1.0 / math.sqrt(C))
    t["meta"] = dict(H=H, W=W, C=C, N=N, G=8, eps=1e-5, heads=1, d=C)
    return t


def attn_layer(seed=2, Hs=64, Ws=64, C=640, N=4, text_len=77, text_dim=2048):
    """Configuration 2: SDXL-shaped self-attention + cross-attention layer (bf16 storage).

    Values are float32 arrays already rounded to bf16.
    """
    L = Hs * Ws
    t = {}
    t["hidden"] = round_bf16(normal(seed, "hidden", (1, L, C)))
    s = 1.0 / math.sqrt(C)
    t["qkv_w"] = round_bf16(normal(seed, "attn1.qkv.w", (3 * C, C), std=s))
    t["o_w"] = round_bf16(normal(seed, "attn1.o.w", (C, C), std=s))
    t["o_b"] = normal(seed, "attn1.o.b", (C,), std=0.02)
    t["k_noise"] = normal(seed, "k_noise", (1, L, C), std=0.02)
    t["v_noise"] = normal(seed, "v_noise", (1, L, C), std=0.02)
    t["text"] = round_bf16(normal(seed, "text", (1, text_len, text_dim)))
    t["q2_w"] = round_bf16(normal(seed, "attn2.q.w", (C, C), std=s))
    t["kv2_w"] = round_bf16(normal(seed, "attn2.kv.w", (2 * C, text_dim), std=1.0 / math.sqrt(text_dim)))
    t["o2_w"] = round_bf16(normal(seed, "attn2.o.w", (C, C), std=s))
    t["o2_b"] = normal(seed, "attn2.o.b", (C,), std=0.02)
    for i in (1, 2):
        t[f"ln{i}_g"] = normal(seed, f"ln{i}.g", (C,), std=0.1, mean=1.0)
        t[f"ln{i}_b"] = normal(seed, f"ln{i}.beta", (C,), std=0.1)
    t["meta"] = dict(L=L, C=C, N=N, heads=C // 64, d=64, text_len=text_len, text_dim=text_dim)
    return t


def attn_core(seed=2, L=4096, C=640, N=4, patch_idx=1, d=64, stale_std=0.02, bf16=True):
    """Q, fresh K/V and stale K/V drawn directly (attention core of configuration 2).

    The full-image K and V are N(0,1); the stale buffers are those plus noise;
    the fresh K/V are the patch's rows of the full-image tensors.
    """
    Lq = L // N
    rnd = round_bf16 if bf16 else (lambda a: a)
    k_full = normal(seed, "k_full", (1, L, C))
    v_full = normal(seed, "v_full", (1, L, C))
    t = {}
    t["q"] = rnd(normal(seed, "q", (1, Lq, C)))
    t["k_fresh"] = rnd(k_full[:, patch_idx * Lq:(patch_idx + 1) * Lq].copy())
    t["v_fresh"] = rnd(v_full[:, patch_idx * Lq:(patch_idx + 1) * Lq].copy())
    t["k_stale"] = rnd(k_full + normal(seed, "k_noise", (1, L, C), std=stale_std))
    t["v_stale"] = rnd(v_full + normal(seed, "v_noise", (1, L, C), std=stale_std))
    t["meta"] = dict(L=L, Lq=Lq, C=C, N=N, patch_idx=patch_idx, heads=C // d, d=d)
    return t


def conv_gn_stage(seed=3, H=128, W=128, C=320, Cout=None, N=4, G=32, bf16=True, stale_std=0.02):
    """Configuration 3: GroupNorm(32) -> 3x3 conv -> SiLU stage on a 128x128x320 latent."""
    Cout = C if Cout is None else Cout
    rnd = round_bf16 if bf16 else (lambda a: a)
    t = {}
    x = normal(seed, "x_full", (1, H, W, C))
    t["x_full"] = rnd(x)
    t["x_stale"] = rnd(x + normal(seed, "stale_noise", (1, H, W, C), std=stale_std))
    t["gamma"] = normal(seed, "gn.gamma", (C,), std=0.1, mean=1.0)
    t["beta"] = normal(seed, "gn.beta", (C,), std=0.1)
    t["conv_w"] = rnd(normal(seed, "conv.w", (Cout, 3, 3, C), std=math.sqrt(2.0 / (9 * C))))
    t["conv_b"] = normal(seed, "conv.b", (Cout,), std=0.02)
    t["meta"] = dict(H=H, W=W, C=C, Cout=Cout, N=N, G=G, eps=1e-5)
    return t


def _draw_weight(seed, name, shape, kind):
    if kind == "w":
        fan_in = 1
        for d in shape[1:]:
            fan_in *= d
        return normal(seed, name, shape, std=1.0 / math.sqrt(fan_in))
    if kind == "b":
        return normal(seed, name, shape, std=0.02)
    if kind == "g":
        return normal(seed, name, shape, std=0.1, mean=1.0)
    if kind == "beta":
        return normal(seed, name, shape, std=0.1)
    raise ValueError(kind)


def unet_weights(cfg, seed=4, threads=8):
    """Random-init UNet parameters in `weight_specs` order.

    Returns a list of (name, array): matrices and conv kernels ("w") as
    uint16 bf16 bit patterns, everything else (biases, norm affine) float32.
    """
    specs = weight_specs(cfg)

    def one(spec):
        name, shape, kind = spec
        a = _draw_weight(seed, name, shape, kind)
        if kind == "w":
            a = to_bf16_bits(a)
        return name, a

    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(one, specs))


def unet_inputs(cfg, seed=4, stale_std=0.02):
    """Latent, embedding and text tensors of a UNet step (configurations 4 and 5)."""
    t = {}
    t["x_prev"] = normal(seed, "x_prev", (1, cfg.H, cfg.W, cfg.in_ch))
    t["x"] = t["x_prev"] + normal(seed, "x_noise", (1, cfg.H, cfg.W, cfg.in_ch), std=stale_std)
    t["emb"] = normal(seed, "emb", (1, cfg.emb_dim))
    t["text"] = round_bf16(normal(seed, "text", (1, cfg.text_len, cfg.text_dim)))
    return t
