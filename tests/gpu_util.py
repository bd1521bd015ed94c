"""Helpers of the GPU parity tests: numpy <-> device tensors, error metrics."""
import numpy as np
import torch

from df_inputs import to_bf16_bits, from_bf16_bits

DEV = "cuda:0"


def dev(a, bf16=False):
    """numpy float array -> device tensor (float32, or bfloat16 from its exact bit pattern)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if bf16:
        bits = to_bf16_bits(a)
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(DEV)
    return torch.from_numpy(a).to(DEV)


def dev_bits(bits):
    """uint16 bf16 bit patterns -> bfloat16 device tensor."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(DEV)


def host(t):
    """device tensor -> float64 numpy (exact)."""
    torch.cuda.synchronize()
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return from_bf16_bits(bits).astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


def rel_l2(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(np.asarray(got, dtype=np.float64) - ref) / max(np.linalg.norm(ref), 1e-30))


def max_rel(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def row_err(got, ref, row_axes=1):
    """Worst row of the tensor: max over rows of ||got_r - ref_r||_2 divided by the RMS row norm of ref.  A row is
    the last `row_axes` axes flattened (one pixel / token for activations [..., C]; `row_axes=2` makes it one image
    row of a [B, R, W, C] tensor with few channels).  Returns (error, index of the worst row)."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64).reshape(ref.shape)
    n = 1
    for d in ref.shape[ref.ndim - row_axes:]:
        n *= d
    r, g = ref.reshape(-1, n), got.reshape(-1, n)
    norms = np.linalg.norm(r, axis=1)
    rms = max(float(np.sqrt(np.mean(norms * norms))), 1e-30)
    e = np.linalg.norm(g - r, axis=1) / rms
    k = int(np.argmax(e))
    return float(e[k]), k


TOL_F32 = 1e-5    # relative L2 error, float32 configurations
TOL_BF16 = 2e-2   # relative L2 error, bf16 storage with float accumulation
# Bounds on single rows and single elements, so that a localised mistake (one row that lost a halo tap, one token
# that attended to the wrong keys) cannot hide inside the whole-tensor norm.  An element of a bf16 result is off by up
# to half a bf16 ulp of its own magnitude (2^-9) plus the accumulated operand rounding, a row by about the
# whole-tensor figure; the bounds leave a factor of two to four over the worst value seen.
ROW_BF16 = 2e-2   # worst row: ||g_r - o_r|| / RMS row norm (single operations; the UNet tests pass 4e-2)
ELT_BF16 = 2e-2   # worst element: max|g - o| / max|o|
ROW_F32 = 1e-5
ELT_F32 = 1e-5


def check(got, ref, bf16, name="", row_axes=1, tol=None, row_tol=None, elt_tol=None, say=None):
    """Asserts the three bounds (whole tensor, worst row, worst element) and returns the whole-tensor error."""
    tol = (TOL_BF16 if bf16 else TOL_F32) if tol is None else tol
    row_tol = (ROW_BF16 if bf16 else ROW_F32) if row_tol is None else row_tol
    elt_tol = (ELT_BF16 if bf16 else ELT_F32) if elt_tol is None else elt_tol
    e, (r, k), m = rel_l2(got, ref), row_err(got, ref, row_axes), max_rel(got, ref)
    if say is not None:
        say("   %s rel_l2 %.3e  worst row %.3e (row %d)  worst element %.3e" % (name, e, r, k, m))
    assert np.isfinite(np.asarray(got, dtype=np.float64)).all(), name
    assert e < tol, (name, "rel_l2", e)
    assert r < row_tol, (name, "worst row", r, k)
    assert m < elt_tol, (name, "worst element", m)
    return e
