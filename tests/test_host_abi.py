"""Host-side checks that need no GPU: the shared library loads and exports every
symbol the header declares, the plan's parameter list equals the layer table's,
and the plan sizing/validation logic behaves."""
import ctypes
import os
import re

import pytest

import paper_2402_19481_amd as df
from df_inputs import unet_table as ut

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "distrifusion.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = sorted(set(re.findall(r"\b(df_[a-z0-9_]+)\s*\(", hdr)))
    assert {"df_attn_displaced", "df_conv3x3_halo", "df_groupnorm_stale", "df_patch_unet_step",
            "df_buffer_refresh"} <= set(names)
    L = ctypes.CDLL(df.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n
    assert df.lib().df_strerror(0) == b"ok" and b"shape" in df.lib().df_strerror(-2)


@pytest.mark.parametrize("kind,H,W,N", [("SDXL", 160, 240, 8), ("SMALL", 16, 8, 2), ("SDXL", 256, 256, 4)])
def test_plan_parameter_list_matches_layer_table(kind, H, W, N):
    cfg = ut.UNetCfg(H=H, W=W, N=N, **getattr(ut, kind))
    got = df.unet_weight_specs(df.make_cfg(cfg))
    want = [(n, tuple(s)) for n, s, _ in ut.weight_specs(cfg)]
    assert got == want


def test_plan_sizes_and_validation():
    L = df.lib()
    cfg = ut.UNetCfg(H=160, W=240, N=8, **ut.SDXL)
    c = df.make_cfg(cfg)
    ws, ss = L.df_unet_workspace_bytes(ctypes.byref(c)), L.df_unet_stale_bytes(ctypes.byref(c))
    # stale state: K and V of 70 self-attention layers dominate
    kv = 2 * 2 * (10 * 9600 * 640 + 60 * 2400 * 1280)
    assert kv < ss < kv * 1.2
    assert 100e6 < ws < 12e9     # arena + two packings (tiled, fragment) of the transformer weights
    bad = df.make_cfg(ut.UNetCfg(H=160, W=240, N=7, **ut.SDXL))       # rows not divisible by the patch count
    assert L.df_unet_num_weights(ctypes.byref(bad)) == -2
    assert L.df_unet_workspace_bytes(ctypes.byref(bad)) == 0
    bad = df.make_cfg(ut.UNetCfg(H=24, W=16, N=2, **ut.SMALL))        # level-1 patch has 6 rows, level 2 has 3: fine
    assert L.df_unet_num_weights(ctypes.byref(bad)) > 0
    bad = df.make_cfg(ut.UNetCfg(H=12, W=16, N=2, **ut.SMALL))        # coarsest level would have 1.5 rows per patch
    assert L.df_unet_num_weights(ctypes.byref(bad)) == -2
