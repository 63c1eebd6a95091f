"""GPU parity of the MFMA GEMM (all three operand layouts, both tile shapes, split contraction, every
epilogue, ragged sizes) against float64 NumPy products of the same float32 inputs."""
import numpy as np
import pytest

from tests.util import dev, host, rel_err, workspace

pytestmark = pytest.mark.gpu


def _run(m, n, k, a_kc, b_kc, epi=0, cfg=-1, splits=0, seed=0, pad=0, alpha=1.0, beta=0.0):
    import torch
    from paper_1507_01239_amd import binding as B
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((m, k)).astype(np.float32)
    Bm = rng.standard_normal((k, n)).astype(np.float32)
    lda = (k if a_kc else m) + pad
    ldb = (k if b_kc else n) + pad
    ldc = n + pad
    a_st = np.zeros((m if a_kc else k, lda), np.float32)
    b_st = np.zeros((n if b_kc else k, ldb), np.float32)
    if a_kc: a_st[:, :k] = A
    else: a_st[:, :m] = A.T
    if b_kc: b_st[:, :k] = Bm.T
    else: b_st[:, :n] = Bm
    bias = rng.standard_normal(n).astype(np.float32)
    aux = rng.random((m, n)).astype(np.float32)
    c0 = rng.standard_normal((m, ldc)).astype(np.float32)
    c = dev(c0)
    ws = workspace(B.mavg_gemm_workspace_bytes(m, n, k, cfg, splits))
    B.mavg_gemm(dev(a_st), lda, a_kc, dev(b_st), ldb, b_kc, c, ldc, m, n, k, epi, dev(bias), dev(aux), n, alpha, beta,
                cfg, splits, ws)
    torch.cuda.synchronize()
    got = host(c)
    v = A.astype(np.float64) @ Bm.astype(np.float64)
    if epi == 1: ref = v + bias
    elif epi == 2: ref = alpha / (1 + np.exp(-(v + bias)))
    elif epi == 3: ref = v * aux * (1.0 - aux)
    elif epi == 4: ref = beta * c0[:, :n].astype(np.float64) + alpha * v
    else: ref = v
    if pad:
        assert np.array_equal(got[:, n:], c0[:, n:])     # nothing written outside the n columns
    return rel_err(got[:, :n], ref)


@pytest.mark.parametrize("a_kc,b_kc", [(1, 1), (1, 0), (0, 0), (0, 1)])
@pytest.mark.parametrize("cfg", [2, 0])
def test_layouts_and_tiles(a_kc, b_kc, cfg):
    # several tiles each way plus ragged tails in m, n and k
    assert _run(200, 328, 148, a_kc, b_kc, cfg=cfg, seed=1) < 2e-6
    assert _run(129, 65, 33, a_kc, b_kc, cfg=cfg, seed=2, pad=4) < 2e-6


@pytest.mark.parametrize("epi", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("splits", [1, 3])
def test_epilogues_with_and_without_split(epi, splits):
    assert _run(96, 160, 200, 1, 1, epi=epi, splits=splits, seed=3, alpha=-0.5, beta=1.0) < 3e-6
    assert _run(70, 132, 260, 0, 0, epi=epi, cfg=0, splits=splits, seed=4, alpha=0.25, beta=0.5) < 3e-6


@pytest.mark.parametrize("a_kc,b_kc", [(1, 1), (1, 0), (0, 0), (0, 1)])
@pytest.mark.parametrize("cfg", [0, 1, 3, 4, 5, 6, 7, 8])
def test_direct_to_lds_variant_and_its_register_staged_twin(a_kc, b_kc, cfg):
    # shapes the direct-to-LDS kernels accept (16-byte aligned rows, contraction a multiple of 16); cfg 0 runs the
    # 64x64 one, cfg 1 forces the register-staged kernel on the same problem, 3 / 4 / 5 are the 128x64, 64x128
    # and 128x128 direct-to-LDS tiles, 6 the 64x64 one with a ring of three LDS stages, 7 the 32x64 tile whose
    # contraction is split four ways inside the workgroup (falls back to 1 below four k-tiles), 8 its 32x32 variant
    # with one wavefront per k-group and no barrier in the loop.  Ragged tile edges in m and n (clamped loads), one
    # to many k-tiles (ring start-up and tail), padded leading dimensions, splits.
    assert _run(200, 328, 144, a_kc, b_kc, cfg=cfg, seed=21) < 2e-6
    assert _run(132, 68, 16, a_kc, b_kc, cfg=cfg, seed=22, pad=4) < 2e-6
    assert _run(64, 64, 32, a_kc, b_kc, cfg=cfg, seed=23) < 2e-6
    assert _run(60, 124, 48, a_kc, b_kc, cfg=cfg, seed=24, pad=8) < 2e-6
    assert _run(256, 192, 1040, a_kc, b_kc, cfg=cfg, seed=25) < 3e-6
    assert _run(128, 256, 640, a_kc, b_kc, cfg=cfg, splits=5, seed=26, epi=2) < 3e-6
    assert _run(4, 4, 80, a_kc, b_kc, cfg=cfg, seed=27) < 2e-6
    # contraction lengths that are not multiples of 16 (a tail after the last whole k-tile), nor of 4
    assert _run(136, 200, 440, a_kc, b_kc, cfg=cfg, seed=28) < 3e-6
    assert _run(72, 100, 90, a_kc, b_kc, cfg=cfg, seed=29, pad=2) < 2e-6
    assert _run(128, 192, 1000, a_kc, b_kc, cfg=cfg, splits=3, seed=30, epi=1) < 3e-6


@pytest.mark.parametrize("epi", [0, 1, 2, 3, 4])
def test_direct_to_lds_epilogues(epi):
    assert _run(200, 264, 64, 0, 0, epi=epi, cfg=5, splits=1, seed=34, alpha=-0.5, beta=1.0) < 3e-6
    assert _run(136, 72, 96, 1, 0, epi=epi, cfg=3, splits=2, seed=35, alpha=0.5, beta=2.0) < 3e-6
    assert _run(96, 160, 208, 1, 1, epi=epi, cfg=0, splits=1, seed=31, alpha=-0.5, beta=1.0) < 3e-6
    assert _run(100, 200, 304, 1, 1, epi=epi, cfg=7, seed=36, alpha=-0.5, beta=1.0) < 3e-6
    assert _run(72, 136, 1024, 1, 0, epi=epi, cfg=7, seed=37, alpha=0.5, beta=2.0) < 3e-6
    assert _run(72, 136, 1024, 1, 1, epi=epi, cfg=8, seed=38, alpha=0.5, beta=2.0) < 3e-6
    assert _run(72, 132, 256, 0, 0, epi=epi, cfg=0, splits=2, seed=32, alpha=0.25, beta=0.5) < 3e-6
    assert _run(100, 64, 96, 1, 0, epi=epi, cfg=0, splits=1, seed=33, alpha=2.0, beta=-1.0) < 3e-6


def test_unaligned_operands_use_the_scalar_path():
    # leading dimensions that are not multiples of 4 (e.g. the paper's 8806-wide output layer)
    assert _run(37, 45, 51, 1, 1, seed=5, pad=1) < 2e-6
    assert _run(37, 46, 50, 1, 0, seed=6, pad=2) < 2e-6
    assert _run(38, 45, 53, 0, 0, seed=7, pad=3) < 2e-6


def test_degenerate_sizes():
    assert _run(1, 1, 1, 1, 1, seed=8) < 1e-6
    assert _run(3, 2, 5, 0, 0, seed=9, splits=4) < 1e-6      # more splits asked for than k tiles exist
    assert _run(64, 64, 16, 1, 0, seed=10) < 1e-6


def test_training_shapes_auto_plan():
    # the full-size layer shapes at minibatch 256 (forward, back-propagation, weight gradient)
    assert _run(256, 2048, 440, 1, 1, epi=2, seed=11) < 3e-6
    assert _run(256, 2048, 2048, 1, 0, epi=3, seed=12) < 3e-6
    assert _run(2048, 440, 256, 0, 0, epi=4, alpha=-0.008, beta=1.0, seed=13) < 3e-6
    assert _run(256, 8000, 2048, 1, 1, epi=1, seed=14) < 3e-6
    assert _run(2048, 2112, 2048, 1, 0, epi=0, seed=15) < 3e-6      # large in all three dimensions: 128x128 tiles


def test_runs_are_bitwise_reproducible():
    import torch
    from paper_1507_01239_amd import binding as B
    rng = np.random.default_rng(0)
    a, b = dev(rng.standard_normal((256, 2048)).astype(np.float32)), dev(rng.standard_normal((512, 2048)).astype(np.float32))
    outs = []
    for _ in range(2):
        c = torch.empty(256, 512, device="cuda")
        ws = workspace(B.mavg_gemm_workspace_bytes(256, 512, 2048, -1, 0))
        B.mavg_gemm(a, 2048, 1, b, 2048, 1, c, 512, 256, 512, 2048, 0, None, None, 0, 1.0, 0.0, -1, 0, ws)
        torch.cuda.synchronize()
        outs.append(host(c))
    assert np.array_equal(outs[0], outs[1])


def test_grouped_launch_of_weight_gradient_shaped_problems():
    # three problems of different sizes in one launch, in the form of a step's weight updates: C <- C + alpha A^T B
    # with both operands row-major over the contraction index (m- and n-contiguous), row sums of A into a vector;
    # one width that is 2 mod 4 read through padded rows
    import torch
    from paper_1507_01239_amd import binding as B
    rng = np.random.default_rng(40)
    n = 96
    shapes = [(200, 72), (64, 136), (86, 52)]          # (m, n_cols): outputs m x n_cols, contraction over n rows
    probs, refs, outs, rows = [], [], [], []
    for (m, nc) in shapes:
        ldd = (m + 3) // 4 * 4
        D = np.zeros((n, ldd), np.float32)
        D[:, :m] = rng.standard_normal((n, m)).astype(np.float32)
        A = rng.standard_normal((n, nc)).astype(np.float32)
        W = rng.standard_normal((m, nc)).astype(np.float32)
        bvec = rng.standard_normal(m).astype(np.float32)
        d_d, a_d, w_d, b_d = dev(D), dev(A), dev(W), dev(bvec)
        probs.append(B.gemm_problem(d_d, ldd, a_d, nc, w_d, nc, m, nc, n, epi=4, alpha=-0.25, beta=1.0,
                                    rowsum_dst=b_d, rowsum_alpha=-0.25, rowsum_beta=1.0, a_pad4=True))
        refs.append((W.astype(np.float64) - 0.25 * D[:, :m].astype(np.float64).T @ A.astype(np.float64),
                     bvec.astype(np.float64) - 0.25 * D[:, :m].astype(np.float64).sum(axis=0)))
        outs.append((w_d, b_d))
        rows.append((d_d, a_d))
    B.mavg_gemm_grouped(probs, 0, 0)
    torch.cuda.synchronize()
    for (w_d, b_d), (Wr, br) in zip(outs, refs):
        assert rel_err(host(w_d), Wr) < 3e-6 and rel_err(host(b_d), br) < 3e-6
