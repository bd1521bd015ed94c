"""The GroupNorm entry point that allocates nothing (df_groupnorm_stale_noalloc) against df_groupnorm_stale.

Both run the same kernels, so the results must agree bit for bit; the difference is where the statistics pass keeps
its partial sums (a fixed array in the library's device image instead of allocated scratch).  Two calls in a row, the
second on a smaller input, so that the array still holds the first call's partials when the second one runs.
"""
import numpy as np
import pytest
import torch

import paper_2402_19481_amd as df
from df_inputs import normal, round_bf16
from oracle import ops
from gpu_util import DEV, check, dev, host

pytestmark = pytest.mark.gpu


def _case(seed, R, W, C, G, N, bf16):
    H = R * N
    full = normal(seed, "full", (1, H, W, C)) * 1.3 + 0.4
    stale = full + normal(seed, "noise", (1, H, W, C), std=0.05)
    if bf16:
        full, stale = round_bf16(full), round_bf16(stale)
    gamma, beta = normal(seed, "g", (C,), std=0.1, mean=1.0), normal(seed, "b", (C,), std=0.1)
    return full, ops.patch_group_sums(stale, G, N).astype(np.float32), gamma, beta


@pytest.mark.parametrize("bf16", [True, False])
def test_noalloc_groupnorm_matches_allocating_entry_point(bf16):
    G, N, patch = 32, 2, 1
    # both shapes take the statistics / finalize / apply kernels (more than 80 K values per group), i.e. use scratch
    shapes = [(72, 128, 320), (66, 128, 320), (4, 8, 64)]        # then a tiny one that needs no scratch at all
    for k, (R, W, C) in enumerate(shapes):
        print("noalloc groupnorm", bf16, R, W, C, flush=True)
        full, st, gamma, beta = _case(70 + k, R, W, C, G, N, bf16)
        xf = full[:, patch * R:(patch + 1) * R]
        x_d, st_d, g_d, b_d = dev(xf, bf16), dev(st), dev(gamma), dev(beta)
        for mode, silu in ((df.GN_SUMS, True), (df.GN_EQ2, False)):
            y_ref, fs_ref = df.groupnorm_stale(x_d, st_d, g_d, b_d, G, patch, N, 1e-5, mode, silu)
            y = torch.full_like(x_d, float("nan"))
            fs = torch.full((1, G, 2), float("nan"), dtype=torch.float32, device=DEV)
            df.groupnorm_stale_noalloc(x_d, st_d, g_d, b_d, G, patch, N, y, fs, 1e-5, mode, silu)
            torch.cuda.synchronize()
            bits = torch.int16 if bf16 else torch.int32
            assert torch.equal(y.view(bits), y_ref.view(bits))
            assert torch.equal(fs.view(torch.int32), fs_ref.view(torch.int32))
            ref, _ = ops.groupnorm_stale(xf, st, gamma, beta, G, patch, N, 1e-5, mode, silu)
            check(host(y), ref, bf16, "noalloc gn %dx%dx%d mode %d" % (R, W, C, mode))


def test_noalloc_groupnorm_rejects_what_does_not_fit():
    # 16 batch items x 64 groups need more partial-sum space than the fixed array holds
    x = torch.zeros(16, 2, 2, 256, device=DEV)
    st = torch.zeros(2, 16, 64, 2, device=DEV)
    g, b = torch.ones(256, device=DEV), torch.zeros(256, device=DEV)
    with pytest.raises(df.DfError):
        df.groupnorm_stale_noalloc(x, st, g, b, 64, 0, 2, torch.empty_like(x), torch.empty(16, 64, 2, device=DEV))
