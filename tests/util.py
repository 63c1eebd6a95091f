"""Shared helpers for the GPU parity tests (no arithmetic of the method lives here)."""
import numpy as np


def rel_err(got, ref) -> float:
    """Norm-wise relative error ||got - ref||_F / ||ref||_F (in float64)."""
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    d = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / d) if d > 0 else float(np.linalg.norm(got))


def dev(a):
    """numpy array -> contiguous CUDA tensor of the same dtype."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def workspace(nbytes):
    import torch
    return torch.empty(int(nbytes) + 256, dtype=torch.uint8, device="cuda")
