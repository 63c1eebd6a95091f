"""GPU parity of replicas_average against the float64 oracle (Sec. 3, eqs. 1-2)."""
import numpy as np
import pytest

import gen
from oracle import averaging
from tests.util import dev, host, rel_err

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("K", [1, 2, 3, 4, 5, 8, 11, 64])
@pytest.mark.parametrize("count,stride", [(8864, 8864), (8864, 9000), (1003, 1004), (3, 4), (4096 * 33 + 2, 4096 * 33 + 4)])
def test_matches_oracle(K, count, stride):
    import torch
    from paper_1507_01239_amd import binding as B
    rng = np.random.default_rng(K * 1000 + count)
    buf = rng.standard_normal((K, stride)).astype(np.float32)
    t = dev(buf)
    B.replicas_average(t, stride, count, K)
    torch.cuda.synchronize()
    out = host(t)
    ref = averaging.average_replicas(buf[:, :count])
    assert rel_err(out[:, :count], ref) < 1e-6            # averaged parameters within 1e-6 relative
    assert np.array_equal(out[:, count:], buf[:, count:])  # gap between replicas untouched
    assert all(np.array_equal(out[0, :count], out[r, :count]) for r in range(K))


@pytest.mark.parametrize("K", [1, 2, 4, 8, 16, 64])
def test_identical_replicas_are_returned_bit_exact_and_averaging_is_idempotent(K):
    import torch
    from paper_1507_01239_amd import binding as B
    v = gen.init_theta(gen.CONFIG_TINY_DIMS, 3, 0.1)
    v[::7] = np.random.default_rng(1).standard_normal(v[::7].size).astype(np.float32)
    t = dev(np.tile(v, (K, 1)))
    B.replicas_average(t, v.size, v.size, K)
    torch.cuda.synchronize()
    assert np.array_equal(host(t), np.tile(v, (K, 1)))
    r = dev(np.random.default_rng(2).standard_normal((K, 4096)).astype(np.float32))
    B.replicas_average(r, 4096, 4096, K)
    once = host(r).copy()
    B.replicas_average(r, 4096, 4096, K)
    torch.cuda.synchronize()
    assert np.array_equal(host(r), once)


def test_empty_is_a_noop():
    import torch
    from paper_1507_01239_amd import binding as B
    t = torch.ones(2, 8, device="cuda")
    B.replicas_average(t, 8, 0, 2)
    torch.cuda.synchronize()
    assert bool((t == 1).all())


def test_full_size_eight_replicas():
    # the benchmarked configuration: 8 replicas of the 440-6x2048-8000 network (38,276,928 parameters each)
    import torch
    from paper_1507_01239_amd import binding as B
    P, K = gen.param_count(gen.CONFIG_FULL_DIMS), 8
    g = torch.Generator(device="cuda").manual_seed(5)
    t = torch.randn(K, P, device="cuda", generator=g) * 0.05
    src = host(t)
    B.replicas_average(t, P, P, K)
    torch.cuda.synchronize()
    out = host(t)
    ref = src.astype(np.float64).sum(axis=0) / K
    assert rel_err(out[0], ref) < 1e-6
    assert all(np.array_equal(out[0], out[r]) for r in range(1, K))
