"""SDXL-shaped UNet layer table as plain data.

The paper names its model only as Stable Diffusion XL (Section 5.1, Models);
the table below is the public SDXL UNet topology restricted to what the
benchmark configurations state: channel levels 320/640/1280, transformer
depths 0/2/10, head dimension 64, cross-attention to 77x2048 text embeddings,
32-group GroupNorm.  It is pinned by the paper's cost figure (Section 3:
6,763 GMACs per step for a 1024x1024 image at classifier-free-guidance batch
2): `count_macs` of this table at a 128x128 latent gives 3380.6 GMACs per
batch item.

Nothing here computes anything of the method; both the oracle and the HIP
path read this table and each builds its own execution from it.
"""
from dataclasses import dataclass


@dataclass(frozen=True)
class UNetCfg:
    H: int                      # full latent height
    W: int                      # full latent width
    N: int = 1                  # number of row patches the image is split into
    in_ch: int = 4
    levels: tuple = (320, 640, 1280)
    depths: tuple = (0, 2, 10)
    head_dim: int = 64
    groups: int = 32
    emb_dim: int = 1280
    text_len: int = 77
    text_dim: int = 2048
    res_per_level: int = 2

    def level_hw(self, level):
        return self.H >> level, self.W >> level


SDXL = dict(levels=(320, 640, 1280), depths=(0, 2, 10), head_dim=64, groups=32,
            emb_dim=1280, text_len=77, text_dim=2048)
# same topology at reduced width, for tests the oracle finishes in seconds
SMALL = dict(levels=(64, 128, 256), depths=(0, 1, 2), head_dim=64, groups=32,
             emb_dim=128, text_len=13, text_dim=96)


def blocks(cfg):
    """Linear list of blocks in execution order.

    Entries (tuples, first element is the kind):
      ("conv_in", name, cin, cout, level)
      ("res", name, cin, cout, level, concat)   concat: pop a skip and concatenate [current, skip] first
      ("xf", name, C, depth, level)
      ("push",)                                  push the current activation on the skip stack
      ("down", name, C, level)                   3x3 stride-2 conv, level -> level+1
      ("up", name, C, level)                     nearest 2x then 3x3 conv, level -> level-1
      ("out", name, cin, cout)                   GroupNorm, SiLU, 3x3 conv to the latent channels
    """
    out = []
    nl = len(cfg.levels)
    c0 = cfg.levels[0]
    out.append(("conv_in", "conv_in", cfg.in_ch, c0, 0))
    out.append(("push",))
    skips = [c0]
    cur = c0
    for li, c in enumerate(cfg.levels):
        for j in range(cfg.res_per_level):
            out.append(("res", f"down{li}.res{j}", cur, c, li, False))
            cur = c
            if cfg.depths[li] > 0:
                out.append(("xf", f"down{li}.xf{j}", c, cfg.depths[li], li))
            out.append(("push",))
            skips.append(cur)
        if li + 1 < nl:
            out.append(("down", f"down{li}.down", cur, li))
            out.append(("push",))
            skips.append(cur)
    lm = nl - 1
    out.append(("res", "mid.res0", cur, cur, lm, False))
    if cfg.depths[lm] > 0:
        out.append(("xf", "mid.xf", cur, cfg.depths[lm], lm))
    out.append(("res", "mid.res1", cur, cur, lm, False))
    for li in reversed(range(nl)):
        c = cfg.levels[li]
        for j in range(cfg.res_per_level + 1):
            sk = skips.pop()
            out.append(("res", f"up{li}.res{j}", cur + sk, c, li, True))
            cur = c
            if cfg.depths[li] > 0:
                out.append(("xf", f"up{li}.xf{j}", c, cfg.depths[li], li))
        if li > 0:
            out.append(("up", f"up{li}.up", cur, li))
    assert not skips
    out.append(("out", "out", cur, cfg.in_ch))
    return out


def weight_specs(cfg):
    """Ordered list of (name, shape, kind) for every parameter tensor.

    kind: "w" weight (std 1/sqrt(fan_in), fan_in = product of all but the
    first dimension), "b" bias (std 0.02), "g" norm scale (1 + 0.1 N(0,1)),
    "beta" norm shift (0.1 N(0,1)).  The fused tensors qkv.w ([3C, C]: rows
    Q, then K, then V), kv.w ([2C, text_dim]: K then V) and ff1.w ([8C, C]:
    value half then gate half) are single parameters of this framework.
    """
    s = []

    def conv(name, cin, cout):
        s.append((name + ".w", (cout, 3, 3, cin), "w"))
        s.append((name + ".b", (cout,), "b"))

    def norm(name, c):
        s.append((name + ".g", (c,), "g"))
        s.append((name + ".beta", (c,), "beta"))

    def lin(name, cin, cout, bias=True):
        s.append((name + ".w", (cout, cin), "w"))
        if bias:
            s.append((name + ".b", (cout,), "b"))

    for b in blocks(cfg):
        kind = b[0]
        if kind == "conv_in":
            conv(b[1], b[2], b[3])
        elif kind == "res":
            _, name, cin, cout, _, _ = b
            norm(name + ".gn1", cin)
            conv(name + ".conv1", cin, cout)
            lin(name + ".emb", cfg.emb_dim, cout)
            norm(name + ".gn2", cout)
            conv(name + ".conv2", cout, cout)
            if cin != cout:
                lin(name + ".sc", cin, cout)
        elif kind == "xf":
            _, name, c, depth, _ = b
            norm(name + ".gn", c)
            lin(name + ".pin", c, c)
            for d in range(depth):
                p = f"{name}.b{d}"
                norm(p + ".ln1", c)
                lin(p + ".attn1.qkv", c, 3 * c, bias=False)
                lin(p + ".attn1.o", c, c)
                norm(p + ".ln2", c)
                lin(p + ".attn2.q", c, c, bias=False)
                lin(p + ".attn2.kv", cfg.text_dim, 2 * c, bias=False)
                lin(p + ".attn2.o", c, c)
                norm(p + ".ln3", c)
                lin(p + ".ff1", c, 8 * c)
                lin(p + ".ff2", 4 * c, c)
            lin(name + ".pout", c, c)
        elif kind in ("down", "up"):
            conv(b[1], b[2], b[2])
        elif kind == "out":
            norm(b[1] + ".gn", b[2])
            conv(b[1] + ".conv", b[2], b[3])
    return s


def num_params(cfg):
    n = 0
    for _, shape, _ in weight_specs(cfg):
        k = 1
        for d in shape:
            k *= d
        n += k
    return n


def count_macs(cfg, n_patches=None):
    """Multiply-accumulates of one patch's share of a step, by class.

    Self-attention counts fresh queries against the full-image key/value set
    (Section 4, Sparse operations), every other layer counts fresh pixels
    only.  n_patches=1 gives the full-image step.
    """
    N = cfg.N if n_patches is None else n_patches
    tot = dict(conv=0, linear=0, self_attn=0, cross_attn=0)

    def px(level):
        h, w = cfg.level_hw(level)
        return (h // N) * w

    def full_px(level):
        h, w = cfg.level_hw(level)
        return h * w

    for b in blocks(cfg):
        kind = b[0]
        if kind == "conv_in":
            tot["conv"] += px(b[4]) * 9 * b[2] * b[3]
        elif kind == "res":
            _, _, cin, cout, lv, _ = b
            tot["conv"] += px(lv) * 9 * (cin * cout + cout * cout)
            tot["linear"] += cfg.emb_dim * cout
            if cin != cout:
                tot["linear"] += px(lv) * cin * cout
        elif kind == "xf":
            _, _, c, depth, lv = b
            p = px(lv)
            tot["linear"] += 2 * p * c * c
            per = p * (3 * c * c + c * c) + p * (c * c + c * c) + p * (c * 8 * c + 4 * c * c)
            per += cfg.text_len * cfg.text_dim * 2 * c
            tot["linear"] += depth * per
            tot["self_attn"] += depth * 2 * p * full_px(lv) * c
            tot["cross_attn"] += depth * 2 * p * cfg.text_len * c
        elif kind == "down":
            tot["conv"] += px(b[3] + 1) * 9 * b[2] * b[2]
        elif kind == "up":
            tot["conv"] += px(b[3] - 1) * 9 * b[2] * b[2]
        elif kind == "out":
            tot["conv"] += px(0) * 9 * b[2] * b[3]
    tot["total"] = sum(tot.values())
    return tot
