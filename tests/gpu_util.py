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


TOL_F32 = 1e-5    # relative L2 error, float32 configurations
TOL_BF16 = 2e-2   # relative L2 error, bf16 storage with float accumulation
