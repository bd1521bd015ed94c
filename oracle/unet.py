"""CPU oracle of one UNet denoising step under displaced patch parallelism (float64).

TEST INFRASTRUCTURE ONLY; shares no code with the HIP path.

A step has two modes (Section 4, Displaced patch parallelism):
  FULL       the first, synchronous step: the ordinary full-image forward.  It
             also leaves, for every spatially mixing layer, the activation the
             next step will see as stale: each 3x3 convolution's input, each
             self-attention's projected keys and values, and each GroupNorm's
             per-patch (sum, sum of squares).
  DISPLACED  one device's view of a later step: only patch `patch_idx` is
             computed; every convolution, self-attention and GroupNorm takes its
             cross-patch context from those stale buffers (oracle.ops), every
             other layer works on the fresh tokens alone.  With refresh the
             patch's own rows of each buffer are overwritten afterwards, which
             is the device-local part of the paper's AllGather.

The network is the SDXL-shaped table of df_inputs.unet_table (data only).
Pins (tests/test_oracle_unet.py): DISPLACED with N=1 equals FULL; with the
buffers a FULL pass leaves on the same input (stale == fresh), every patch's
DISPLACED output equals its rows of the FULL output and the patches tile it;
the table's MAC count matches the paper's 6,763 GMACs.

PARITY UNPINNED: the wiring of _resblock / _transformer / unet_step (order of
the skip concatenation, norm epsilons, SiLU on the embedding, where residuals
enter).  The paper names the network ("SDXL") without defining its wiring and
prints no value of the chain; the pins above hold for any wiring of the same
shapes.  The layer operations themselves (oracle.ops) are pinned.
"""
import numpy as np

from . import ops

FULL = 0
DISPLACED = 1


class _Ctx:
    """Spatially mixing layers of one step; per-token layers do not need it."""

    def __init__(self, cfg, mode, stale, patch_idx, refresh, stat_mode, split_axis=1):
        self.cfg, self.mode, self.stale = cfg, mode, stale
        self.i, self.refresh, self.stat_mode = patch_idx, refresh, stat_mode
        self.N = cfg.N
        self.axis = split_axis          # 1: horizontal strips (rows), 2: vertical strips (columns)

    def conv(self, name, x, w, b, stride=1):
        key = name + ".in"
        if self.mode == FULL:
            self.stale[key] = np.array(x, dtype=np.float64)
            return ops.conv3x3_full(x, w, b, stride)
        y = ops.conv3x3_halo(x, self.stale[key], w, b, self.i, self.N, stride, split_axis=self.axis)
        if self.refresh:
            ops.buffer_refresh(self.stale[key], x, self.i, self.N, axis=self.axis)
        return y

    def groupnorm(self, name, x, gamma, beta, eps, silu):
        key = name + ".stats"
        G = self.cfg.groups
        if self.mode == FULL:
            self.stale[key] = ops.patch_group_sums(x, G, self.N, axis=self.axis)
            y, _ = ops.groupnorm_stale(x, ops.group_sums(x, G)[None], gamma, beta, G, 0, 1, eps, ops.STAT_SUMS, silu)
            return y
        y, fresh = ops.groupnorm_stale(x, self.stale[key], gamma, beta, G, self.i, self.N, eps, self.stat_mode, silu)
        if self.refresh:
            self.stale[key][self.i] = fresh
        return y

    def self_attention(self, name, q, k, v, heads, hw):
        """q, k, v: the fresh tokens [B, Lq, C] in row-major pixel order of the patch; hw: the full token grid."""
        if self.mode == FULL:
            self.stale[name + ".k"] = np.array(k, dtype=np.float64)
            self.stale[name + ".v"] = np.array(v, dtype=np.float64)
            return ops.attention_dense(q, k, v, heads)
        ks, vs = self.stale[name + ".k"], self.stale[name + ".v"]
        o = ops.attn_displaced(q, k, v, ks, vs, heads, self.i, self.N, split_axis=self.axis, hw=hw)
        if self.refresh:
            if self.axis == 1:
                ops.buffer_refresh(ks, k, self.i, self.N)
                ops.buffer_refresh(vs, v, self.i, self.N)
            else:               # the strip's tokens go to its columns of the [B, H, W, C] view of the buffers
                B, C = k.shape[0], k.shape[-1]
                H, W = hw
                for buf, new in ((ks, k), (vs, v)):
                    ops.buffer_refresh(buf.reshape(B, H, W, C), np.asarray(new).reshape(B, H, W // self.N, C), self.i,
                                       self.N, axis=2)
        return o


def _resblock(ctx, P, name, x, emb, cin, cout):
    h = ctx.groupnorm(name + ".gn1", x, P[name + ".gn1.g"], P[name + ".gn1.beta"], 1e-5, True)
    h = ctx.conv(name + ".conv1", h, P[name + ".conv1.w"], P[name + ".conv1.b"])
    e = ops.linear(ops.silu(emb), P[name + ".emb.w"], P[name + ".emb.b"])          # [B, cout]
    h = h + e[:, None, None, :]
    h = ctx.groupnorm(name + ".gn2", h, P[name + ".gn2.g"], P[name + ".gn2.beta"], 1e-5, True)
    h = ctx.conv(name + ".conv2", h, P[name + ".conv2.w"], P[name + ".conv2.b"])
    sc = x if cin == cout else ops.linear(x, P[name + ".sc.w"], P[name + ".sc.b"])
    return sc + h


def _transformer(ctx, P, name, x, text, C, depth):
    cfg = ctx.cfg
    heads = C // cfg.head_dim
    B, R, W, _ = x.shape
    # the full token grid of this level (x holds the whole image, or one strip of it)
    hw = (R, W) if ctx.mode == FULL else ((R * ctx.N, W) if ctx.axis == 1 else (R, W * ctx.N))
    h = ctx.groupnorm(name + ".gn", x, P[name + ".gn.g"], P[name + ".gn.beta"], 1e-6, False)
    h = ops.linear(h.reshape(B, R * W, C), P[name + ".pin.w"], P[name + ".pin.b"])
    for d in range(depth):
        p = f"{name}.b{d}"
        n = ops.layernorm(h, P[p + ".ln1.g"], P[p + ".ln1.beta"])
        qkv = ops.linear(n, P[p + ".attn1.qkv.w"])
        a = ctx.self_attention(p + ".attn1", qkv[..., :C], qkv[..., C:2 * C], qkv[..., 2 * C:], heads, hw)
        h = h + ops.linear(a, P[p + ".attn1.o.w"], P[p + ".attn1.o.b"])
        n = ops.layernorm(h, P[p + ".ln2.g"], P[p + ".ln2.beta"])
        q = ops.linear(n, P[p + ".attn2.q.w"])
        kv = ops.linear(text, P[p + ".attn2.kv.w"])
        a = ops.attention_dense(q, kv[..., :C], kv[..., C:], heads)
        h = h + ops.linear(a, P[p + ".attn2.o.w"], P[p + ".attn2.o.b"])
        n = ops.layernorm(h, P[p + ".ln3.g"], P[p + ".ln3.beta"])
        f = ops.geglu(ops.linear(n, P[p + ".ff1.w"], P[p + ".ff1.b"]))
        h = h + ops.linear(f, P[p + ".ff2.w"], P[p + ".ff2.b"])
    h = ops.linear(h, P[name + ".pout.w"], P[name + ".pout.b"])
    return x + h.reshape(B, R, W, C)


class Params:
    """Name -> float64 view of the parameter list (matrices arrive as bf16 bit patterns)."""

    def __init__(self, weights):
        self._w = dict(weights)

    def __getitem__(self, name):
        a = self._w[name]
        if a.dtype == np.uint16:
            a = (a.astype(np.uint32) << np.uint32(16)).view(np.float32)
        return a.astype(np.float64)


def unet_step(cfg, blocks, weights, x, emb, text, stale, patch_idx=0, mode=FULL, refresh=True,
              stat_mode=ops.STAT_SUMS, trace=None, resume=None, on_block=None, split_axis=1):
    """One UNet forward.

    x: FULL [B,H,W,in_ch]; DISPLACED [B,H/N,W,in_ch] (the patch's rows), or [B,H,W/N,in_ch] with split_axis=2
    (vertical strips; Section 5.1, Baselines).
    emb [B,emb_dim], text [B,text_len,text_dim].  `stale` is a dict that FULL
    fills and DISPLACED reads (and refreshes in place).  `blocks` is
    df_inputs.unet_table.blocks(cfg).  Returns the predicted noise for the rows
    of x.  `trace`, if a dict, receives the output of every block by name.
    Long runs can be interrupted and continued: `on_block(n, h, skips)` is called after the n-th entry of the block
    list with the activation and the pending skip connections, and `resume=(n, h, skips)` starts after that entry
    (with `stale` as it stood then).  Neither changes what is computed.
    """
    P = weights if isinstance(weights, Params) else Params(weights)
    ctx = _Ctx(cfg, mode, stale, patch_idx, refresh, stat_mode, split_axis)
    x = np.asarray(x, dtype=np.float64)
    emb = np.asarray(emb, dtype=np.float64)
    text = np.asarray(text, dtype=np.float64)
    skips = []
    h = x
    start = 0
    if resume is not None:
        start, h, skips = resume[0], np.asarray(resume[1], dtype=np.float64), list(resume[2])
    for bi, b in enumerate(blocks):
        if bi < start:
            continue
        kind = b[0]
        if kind == "conv_in":
            h = ctx.conv(b[1], h, P[b[1] + ".w"], P[b[1] + ".b"])
        elif kind == "push":
            skips.append(h)
        elif kind == "res":
            _, name, cin, cout, _, concat = b
            if concat:
                h = np.concatenate([h, skips.pop()], axis=-1)
            h = _resblock(ctx, P, name, h, emb, cin, cout)
        elif kind == "xf":
            _, name, C, depth, _ = b
            h = _transformer(ctx, P, name, h, text, C, depth)
        elif kind == "down":
            h = ctx.conv(b[1], h, P[b[1] + ".w"], P[b[1] + ".b"], stride=2)
        elif kind == "up":
            h = ctx.conv(b[1], ops.upsample_nearest2x(h), P[b[1] + ".w"], P[b[1] + ".b"])
        elif kind == "out":
            h = ctx.groupnorm(b[1] + ".gn", h, P[b[1] + ".gn.g"], P[b[1] + ".gn.beta"], 1e-5, True)
            h = ctx.conv(b[1] + ".conv", h, P[b[1] + ".conv.w"], P[b[1] + ".conv.b"])
        if trace is not None and kind != "push":
            trace[b[1]] = h
        if on_block is not None:
            on_block(bi + 1, h, skips)
    return h


def euler_update(x, eps, sigma, sigma_next):
    """Element-wise sampler update (Section 3, Eq. 1) for an Euler step on the sigma ladder."""
    return np.asarray(x, dtype=np.float64) + (sigma_next - sigma) * np.asarray(eps, dtype=np.float64)
