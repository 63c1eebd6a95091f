"""rbm_cd1_step_static (the CD-1 step with its scratch in a static device array inside the library, for callers
that cannot allocate) against rbm_cd1_step with a caller-provided workspace: same kernels, so the updated
parameters, momentum buffers and the reconstruction error must agree bit for bit.  Two calls in a row on the one
static array, the second on a smaller problem of a different kind, then the first again."""
import numpy as np
import pytest

import gen
from tests.util import dev, host, workspace

pytestmark = pytest.mark.gpu


def _case(V, H, n, vis, flags, lr, seed, step):
    W, a, c = gen.rbm_params(V, H, seed, 0, 0.1)
    rng = np.random.default_rng(seed)
    mom = [rng.standard_normal(t.shape).astype(np.float32) * 0.01 for t in (W, a, c)]
    V0 = gen.features_speech_like(n, V, seed, 0, step) if vis == 1 else gen.rbm_binary_input(n, V, seed, step)
    return [W, a, c] + mom, V0


def _run(static, V, H, n, vis, flags, lr, seed, step):
    import torch
    from paper_1507_01239_amd import binding as B
    params, V0 = _case(V, H, n, vis, flags, lr, seed, step)
    t = [dev(p) for p in params]
    err = torch.full((1,), -1.0, device="cuda")
    if static:
        B.rbm_cd1_step_static(V, H, vis, *t, dev(V0), n, lr, 0.9, seed, step, 2, flags, err)
    else:
        B.rbm_cd1_step(V, H, vis, *t, dev(V0), n, lr, 0.9, seed, step, 2, flags, err, workspace(B.rbm_workspace_bytes(V, H, n)))
    torch.cuda.synchronize()
    return [host(x).copy() for x in t] + [host(err).copy()]


def test_static_scratch_cd1_matches_the_workspace_entry_point_on_consecutive_calls():
    cases = [(440, 2048, 256, 1, 0, 0.01, 71, 0),       # Gaussian visibles, the first pretraining RBM's shape
             (61, 35, 50, 0, 1, 0.4, 72, 1),            # smaller, ragged, Bernoulli visibles with sampled reconstruction
             (440, 2048, 256, 1, 0, 0.01, 71, 0)]       # the first one again, over the second's leftovers
    for V, H, n, vis, flags, lr, seed, step in cases:
        got = _run(True, V, H, n, vis, flags, lr, seed, step)
        want = _run(False, V, H, n, vis, flags, lr, seed, step)
        for name, g, w in zip(("W", "a", "c", "MW", "Ma", "Mc", "recon_err"), got, want):
            assert np.all(np.isfinite(g)), name
            assert np.array_equal(g, w), (V, H, n, name)
        assert got[-1][0] > 0.0


def test_static_scratch_rejects_what_does_not_fit_without_launching():
    import torch
    from paper_1507_01239_amd import binding as B
    assert B.rbm_workspace_bytes(2048, 2048, 512) - 256 <= B.RBM_STATIC_SCRATCH_BYTES
    assert B.rbm_workspace_bytes(2048, 2048, 1024) - 256 > B.RBM_STATIC_SCRATCH_BYTES
    A = 1 << 20          # fake aligned addresses: a call that is rejected never dereferences them
    rc = B.lib.rbm_cd1_step_static(2048, 2048, 0, A, A, A, A, A, A, A, 1024, 0.1, 0.9, 1, 0, 0, 0, None, None)
    assert rc == B.E_WORKSPACE
    assert B.lib.rbm_cd1_step_static(8, 4, 0, None, A, A, A, A, A, A, 4, 0.1, 0.9, 1, 0, 0, 0, None, None) == B.E_NULL
