"""Shared helpers of the GPU parity tests: host <-> device plumbing and the error metric."""
import numpy as np


def rel_fro(got, ref):
    """||got - ref||_F / ||ref||_F ; if ref is all zero, got must be too."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    n = np.linalg.norm(ref)
    if n == 0:
        return 0.0 if np.linalg.norm(got) == 0 else np.inf
    return float(np.linalg.norm(got - ref) / n)


def dev_bf16(a):
    """float32 numpy array holding bf16-representable values -> bf16 cuda tensor."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).cuda()


def dev_f32(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def host(t):
    """cuda tensor (bf16 or fp32) -> float64 numpy."""
    return t.float().cpu().numpy().astype(np.float64)
