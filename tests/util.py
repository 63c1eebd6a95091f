"""Shared helpers for the GPU parity tests (no arithmetic of the method lives here)."""
import numpy as np


def rel_err(got, ref) -> float:
    """Norm-wise relative error ||got - ref||_F / ||ref||_F (in float64)."""
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    d = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / d) if d > 0 else float(np.linalg.norm(got))


def max_err(got, ref) -> float:
    """Largest element-wise error, each element's error measured against its own magnitude plus the tensor's root
    mean square: max_i |got_i - ref_i| / (|ref_i| + rms(ref)).

    The norm-wise error averages over a tensor; this one is the check that no single element is far off (one
    typical element of a 2048 x 2048 matrix wrong by a tenth of its value reads 0.05 here and 5e-5 norm-wise).
    The element's own magnitude is in the scale because rounding errors grow with the terms that were summed:
    in a heavy-tailed tensor (the output layer's rows of the frequent classes under a Zipf prior) a few elements
    are fifty times the root mean square, and so are their rounding errors."""
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    if rms == 0.0:
        return float(np.abs(got).max())
    return float((np.abs(got - ref) / (np.abs(ref) + rms)).max())


def check_close(got, ref, tol, what="", max_factor=20.0):
    """Assert the norm-wise relative error below tol AND the largest element-wise error (max_err) below
    max_factor * tol.  Random rounding errors of a few million elements reach 5 to 6 standard deviations; a factor
    of 20 leaves room for that and still catches a single element that is off by 4 % of its own value at
    tol = 1e-3, 0.4 % at 1e-4.  Returns both figures."""
    r, m = rel_err(got, ref), max_err(got, ref)
    assert r < tol, f"{what}: norm-wise relative error {r:.3e} >= {tol:.1e} (largest element error {m:.3e})"
    assert m < max_factor * tol, f"{what}: largest element error {m:.3e} >= {max_factor * tol:.1e} (norm-wise {r:.3e})"
    return r, m


def dev(a):
    """numpy array -> contiguous CUDA tensor of the same dtype."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def workspace(nbytes):
    import torch
    return torch.empty(int(nbytes) + 256, dtype=torch.uint8, device="cuda")
