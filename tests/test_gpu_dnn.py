"""GPU parity of dnn_forward / dnn_backward_update (+ replicas_average) against the float64 oracle.

Tolerances are those fixed for this build: per-step activations and gradients 1e-4 relative
(norm-wise per tensor), parameters after 50 steps 1e-3 relative, averaged parameters 1e-6 relative.
Next to every norm-wise figure the largest element-wise error is bounded too (tests.util.check_close)."""
import numpy as np
import pytest

import gen
from oracle import averaging, dnn
from tests.util import check_close, dev, host, rel_err, workspace

pytestmark = pytest.mark.gpu

ACT_TOL, GRAD_TOL, PARAM_TOL = 1e-4, 1e-4, 1e-3


class Gpu:
    """k replicas of one network on the device, driven through the C ABI."""

    def __init__(self, dims, k, n, theta0, flags=None, hidden_act=0):
        import torch
        from paper_1507_01239_amd import binding as B
        self.B, self.torch = B, torch
        self.dims, self.k, self.n = dims, k, n
        self.shape = B.Shape(dims, hidden_act)
        self.P = B.mavg_param_count(self.shape)
        self.stride = (self.P + 63) // 64 * 64
        self.act_stride = (B.mavg_act_count(self.shape, n) + 63) // 64 * 64
        self.flags = B.MEAN_GRAD if flags is None else flags
        self.theta = torch.zeros(k, self.stride, device="cuda")
        self.theta[:, :self.P] = dev(theta0)[None, :]
        self.acts = torch.empty(k, self.act_stride, device="cuda")
        self.ws = workspace(B.mavg_workspace_bytes(self.shape, n, k, self.flags))
        self.loss = torch.zeros(k, device="cuda")

    def forward(self, X):
        """X: k x n x d0 numpy."""
        self.x = dev(X.reshape(self.k, -1))
        self.B.dnn_forward(self.shape, self.k, self.theta, self.stride, self.x, self.x.shape[1], self.n, self.acts,
                           self.act_stride, self.ws)

    def backward(self, Y, lr):
        self.y = dev(Y.reshape(self.k, -1).astype(np.int32))
        self.B.dnn_backward_update(self.shape, self.k, self.theta, self.stride, self.x, self.x.shape[1], self.y,
                                   self.y.shape[1], self.n, self.acts, self.act_stride, lr, self.flags, self.loss, self.ws)

    def step(self, X, Y, lr):
        self.forward(X)
        self.backward(Y, lr)

    def average(self):
        self.B.replicas_average(self.theta, self.stride, self.P, self.k)

    def params(self):
        self.torch.cuda.synchronize()
        return host(self.theta[:, :self.P])

    def activations(self, r=0):
        self.torch.cuda.synchronize()
        a = host(self.acts[r])
        out, off = [], 0
        for d in self.dims[1:]:
            out.append(a[off:off + self.n * d].reshape(self.n, d))
            off += self.n * d
        return out


def check_tensors(got_flat, ref_flat, dims, tol, what):
    """Per weight matrix and bias vector: norm-wise and element-wise bounds.  Returns the worst pair seen."""
    worst = (0.0, 0.0)
    got = dnn.unpack(np.asarray(got_flat, np.float64), dims)
    ref = dnn.unpack(np.asarray(ref_flat, np.float64), dims)
    for l, ((Wg, bg), (Wr, br)) in enumerate(zip(got, ref), start=1):
        for name, g, r in (("W", Wg, Wr), ("b", bg, br)):
            e = check_close(g, r, tol, f"{what} {name}{l}")
            worst = (max(worst[0], e[0]), max(worst[1], e[1]))
    return worst


def check_acts(gpu_acts, ref_acts, tol, what):
    for l, (a_gpu, a_ref) in enumerate(zip(gpu_acts, ref_acts), start=1):
        check_close(a_gpu, a_ref, tol, f"{what} A{l}")


def _tiny_shards(seed, K, T, n, dims):
    return [[(gen.features_iid(n, dims[0], seed, k, t), gen.labels_uniform(n, dims[-1], seed, k, t))
             for t in range(T)] for k in range(K)]


def test_config1_tiny_four_replicas_averaged_every_two():
    # 40-64-64-32, minibatch 32, lr 0.1, 4 replicas, averaging every 2 minibatches, 8 minibatches per replica
    dims, K, T, n, lr, n_avg, seed = gen.CONFIG_TINY_DIMS, 4, 8, 32, 0.1, 2, 7
    theta0 = gen.init_theta(dims, seed, 0.1)
    shards = _tiny_shards(seed, K, T, n, dims)
    trace = []
    ref_thetas, ref_losses = averaging.train_with_averaging(theta0, dims, shards, lr, n_avg, trace=trace)
    g = Gpu(dims, K, n, theta0)
    for t in range(T):
        X = np.stack([shards[k][t][0] for k in range(K)])
        Y = np.stack([shards[k][t][1] for k in range(K)])
        g.forward(X)
        if t == 0:
            check_acts(g.activations(2), dnn.forward(theta0, dims, X[2]), ACT_TOL, "replica 2, first minibatch")
        g.backward(Y, lr)
        losses = host(g.loss)
        assert np.allclose(losses, ref_losses[:, t], rtol=1e-4)
        if (t + 1) % n_avg == 0:
            g.average()
        check_close(g.params(), trace[t], PARAM_TOL, f"parameters after minibatch {t}")
    th = g.params()
    for k in range(K):
        check_tensors(th[k], ref_thetas[k], dims, PARAM_TOL, f"replica {k}")
    assert all(np.array_equal(th[0], th[r]) for r in range(K))     # every replica holds the average


def test_averaging_every_update_equals_gradient_averaging_on_gpu():
    # Sec. 3: K replicas, one step each on its own shard, then averaging == one step on the concatenated batch
    dims, K, n, lr, seed = gen.CONFIG_TINY_DIMS, 4, 32, 0.1, 9
    theta0 = gen.init_theta(dims, seed, 0.1)
    shards = _tiny_shards(seed, K, 1, n, dims)
    X = np.stack([shards[k][0][0] for k in range(K)])
    Y = np.stack([shards[k][0][1] for k in range(K)])
    g = Gpu(dims, K, n, theta0)
    g.step(X, Y, lr)
    g.average()
    one = Gpu(dims, 1, K * n, theta0)
    one.step(X.reshape(1, K * n, -1), Y.reshape(1, -1), lr)
    assert rel_err(g.params()[0], one.params()[0]) < 1e-6


@pytest.mark.parametrize("mean", [True, False])
def test_per_step_gradient_and_activations_tiny_ragged(mean):
    # widths and minibatch that are not multiples of any tile, incl. an odd output layer
    dims, n = (44, 72, 36, 52), 37
    rng = np.random.default_rng(3)
    theta0 = (rng.standard_normal(gen.param_count(dims)) * 0.3).astype(np.float32)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    y = rng.integers(0, dims[-1], n).astype(np.int32)
    from paper_1507_01239_amd import binding as B
    g = Gpu(dims, 1, n, theta0, flags=B.MEAN_GRAD if mean else 0)
    lr = 4.0 if mean else 0.125
    g.step(X[None], y[None], lr)
    check_acts(g.activations(0), dnn.forward(theta0, dims, X), ACT_TOL, "ragged")
    grad_ref, loss_ref = dnn.gradient(theta0, dims, X, y, mean_grad=mean)
    grad_gpu = (theta0.astype(np.float64) - g.params()[0].astype(np.float64)) / lr
    check_tensors(grad_gpu, grad_ref, dims, GRAD_TOL, "gradient")
    assert abs(host(g.loss)[0] - loss_ref) < 1e-4 * abs(loss_ref)


def test_unaligned_widths_paper_like_output():
    # widths that are not multiples of 4 anywhere (the paper's own output layer has 8806 units)
    dims, n = (10, 13, 7, 9), 5
    rng = np.random.default_rng(4)
    theta0 = (rng.standard_normal(gen.param_count(dims)) * 0.4).astype(np.float32)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    y = rng.integers(0, dims[-1], n).astype(np.int32)
    g = Gpu(dims, 1, n, theta0)
    g.step(X[None], y[None], 2.0)
    ref, _, acts_ref = dnn.sgd_step(theta0, dims, X, y, 2.0)
    check_acts(g.activations(0), acts_ref, ACT_TOL, "unaligned")
    check_tensors(g.params()[0], ref, dims, 1e-5, "parameters")


def test_zero_learning_rate_leaves_parameters_bit_identical():
    dims, n = gen.CONFIG_TINY_DIMS, 32
    theta0 = gen.init_theta(dims, 1, 0.1)
    g = Gpu(dims, 2, n, theta0)
    X = np.stack([gen.features_iid(n, 40, 1, k, 0) for k in range(2)])
    Y = np.stack([gen.labels_uniform(n, 32, 1, k, 0) for k in range(2)])
    g.step(X, Y, 0.0)
    assert np.array_equal(g.params()[0], theta0) and np.array_equal(g.params()[1], theta0)


def _full_batch(seed, replica, t, n):
    dims = gen.CONFIG_FULL_DIMS
    return (gen.features_speech_like(n, dims[0], seed, replica, t), gen.labels_zipf(n, dims[-1], seed, replica, t))


def test_config2_full_size_fifty_steps():
    # 440-6x2048-8000, minibatch 256, lr 0.008, mean gradient: activations and gradient of the first step,
    # parameters after 50 steps
    dims, n, lr, seed, T = gen.CONFIG_FULL_DIMS, 256, 0.008, 21, 50
    theta0 = gen.init_theta(dims, seed, 0.05)
    g = Gpu(dims, 1, n, theta0)
    ref = theta0.astype(np.float64)
    for t in range(T):
        X, y = _full_batch(seed, 0, t, n)
        g.forward(X[None])
        if t in (0, T - 1):
            check_acts(g.activations(0), dnn.forward(ref, dims, X), ACT_TOL if t == 0 else PARAM_TOL, f"minibatch {t}")
        g.backward(y[None], lr)
        ref, loss_ref, _ = dnn.sgd_step(ref, dims, X, y, lr)
        if t in (0, T - 1):
            assert abs(host(g.loss)[0] - loss_ref) < 1e-3 * abs(loss_ref)
    th = g.params()[0]
    assert rel_err(th, ref) < PARAM_TOL
    worst = check_tensors(th, ref, dims, PARAM_TOL, "after 50 steps")       # every weight matrix AND every bias vector
    print(f"50 steps: worst per-tensor relative error {worst[0]:.2e}, worst element {worst[1]:.2e}")


@pytest.mark.parametrize("n", [128, 256, 512, 1024])
def test_full_size_first_step_gradient(n):
    # the minibatch sizes of the averaging sweep: each takes different tile plans (contraction splits, ring depth)
    dims, seed = gen.CONFIG_FULL_DIMS, 22
    theta0 = gen.init_theta(dims, seed, 0.05)
    X, y = _full_batch(seed, 0, 0, n)
    lr = 16.0       # a power of two large enough that (theta - theta')/lr resolves the gradient in float32
    g = Gpu(dims, 1, n, theta0)
    g.step(X[None], y[None], lr)
    grad_ref, _ = dnn.gradient(theta0, dims, X, y, mean_grad=True)
    grad_gpu = (theta0.astype(np.float64) - g.params()[0].astype(np.float64)) / lr
    check_tensors(grad_gpu, grad_ref, dims, GRAD_TOL, f"gradient at minibatch {n}")


def test_config3_eight_full_size_replicas_two_averaging_periods():
    # 8 replicas resident on the device, each on its own shard, averaged every 2 minibatches (minibatch 128)
    dims, K, n, lr, n_avg, seed, T = gen.CONFIG_FULL_DIMS, 8, 128, 0.008, 2, 23, 4
    theta0 = gen.init_theta(dims, seed, 0.05)
    shards = [[_full_batch(seed, k, t, n) for t in range(T)] for k in range(K)]
    ref, ref_losses = averaging.train_with_averaging(theta0, dims, shards, lr, n_avg)
    g = Gpu(dims, K, n, theta0)
    for t in range(T):
        X = np.stack([shards[k][t][0] for k in range(K)])
        Y = np.stack([shards[k][t][1] for k in range(K)])
        g.step(X, Y, lr)
        assert np.allclose(host(g.loss), ref_losses[:, t], rtol=1e-3)
        if (t + 1) % n_avg == 0:
            g.average()
    th = g.params()
    check_tensors(th[0], ref[0], dims, PARAM_TOL, "averaged parameters after 4 minibatches")
    assert all(np.array_equal(th[0], th[r]) for r in range(1, K))


def test_full_size_activations_two_replicas_minibatch_512():
    # forward pass at full size through the grouped (2-replica) launch: every layer's activations per replica
    dims, n, K, seed = gen.CONFIG_FULL_DIMS, 512, 2, 24
    theta0 = gen.init_theta(dims, seed, 0.05)
    Xs = np.stack([_full_batch(seed, k, 0, n)[0] for k in range(K)])
    g = Gpu(dims, K, n, theta0)
    g.forward(Xs)
    for k in range(K):
        check_acts(g.activations(k), dnn.forward(theta0, dims, Xs[k]), ACT_TOL, f"replica {k}")


def test_single_frame_minibatch_and_many_replicas():
    # degenerate sizes: one frame per minibatch; 16 replicas of a small ragged network in one launch
    dims, seed = [12, 9, 7, 5], 31        # (replica strides of the inputs must be multiples of 4 floats)
    theta0 = gen.init_theta(dims, seed, 0.3)
    for K, n in ((1, 1), (16, 1), (16, 3)):
        X = np.stack([gen.features_iid(n, dims[0], seed, k, 0) for k in range(K)])
        Y = np.stack([gen.labels_uniform(n, dims[-1], seed, k, 0) for k in range(K)])
        g = Gpu(dims, K, n, theta0)
        g.step(X, Y, 0.5)
        th = g.params()
        for k in range(K):
            ref, loss, acts = dnn.sgd_step(theta0, dims, X[k], Y[k], 0.5)
            assert rel_err(th[k], ref) < 1e-5
            assert abs(float(host(g.loss)[k]) - loss) < 1e-4 * max(1.0, abs(loss))


@pytest.mark.parametrize("dims,n", [([13, 11, 9, 7, 6], 10), ([440, 256, 192, 500], 96)])
def test_tanh_hidden_units_activations_gradient_and_five_steps(dims, n):
    # the variant nonlinearity (tanh hidden units): per-step activations and gradient, then a short trajectory
    seed = 41
    theta0 = gen.init_theta(dims, seed, 0.2)
    X = gen.features_iid(n, dims[0], seed, 0, 0)
    y = gen.labels_uniform(n, dims[-1], seed, 0, 0)
    lr = 4.0
    g = Gpu(dims, 1, n, theta0, hidden_act=1)
    g.step(X[None], y[None], lr)
    check_acts(g.activations(0), dnn.forward(theta0, dims, X, hidden="tanh"), ACT_TOL, "tanh")
    grad_ref, loss_ref = dnn.gradient(theta0, dims, X, y, mean_grad=True, hidden="tanh")
    grad_gpu = (theta0.astype(np.float64) - g.params()[0].astype(np.float64)) / lr
    check_tensors(grad_gpu, grad_ref, dims, GRAD_TOL, "tanh gradient")
    assert abs(float(host(g.loss)[0]) - loss_ref) < 1e-4 * abs(loss_ref)
    g2 = Gpu(dims, 1, n, theta0, hidden_act=1)
    ref = theta0.astype(np.float64)
    for t in range(5):
        Xt = gen.features_iid(n, dims[0], seed, 0, t)
        yt = gen.labels_uniform(n, dims[-1], seed, 0, t)
        g2.step(Xt[None], yt[None], 0.05)
        ref, _, _ = dnn.sgd_step(ref, dims, Xt, yt, 0.05, hidden="tanh")
    check_tensors(g2.params()[0], ref, dims, PARAM_TOL, "tanh, five steps")


def _speech_batch(dims, seed, replica, t, n):
    return (gen.features_speech_like(n, dims[0], seed, replica, t), gen.labels_zipf(n, dims[-1], seed, replica, t))


@pytest.mark.parametrize("dims,n,K", [((44, 70, 38, 86), 37, 2), ((440, 256, 8806), 128, 1), ((440, 256, 8806), 1024, 2)])
def test_output_width_two_mod_four_on_the_direct_load_kernels(dims, n, K):
    # Sec. 5.1's output layer has 8806 units: a width that is 2 mod 4.  With 16 or more rows per minibatch the
    # weight-gradient launch reads delta_L (rows padded to a multiple of 4 inside the workspace) with the
    # direct-to-LDS kernel, up to the padding columns that the output-error kernel never writes, and updates the
    # bias through the fused row sums.  First step: activations and gradient per tensor; then five steps.
    seed = 51
    theta0 = gen.init_theta(dims, seed, 0.1)
    X = np.stack([_speech_batch(dims, seed, k, 0, n)[0] for k in range(K)])
    Y = np.stack([_speech_batch(dims, seed, k, 0, n)[1] for k in range(K)])
    lr = 16.0
    g = Gpu(dims, K, n, theta0)
    g.step(X, Y, lr)
    th = g.params()
    for k in range(K):
        check_acts(g.activations(k), dnn.forward(theta0, dims, X[k]), ACT_TOL, f"replica {k}")
        grad_ref, loss_ref = dnn.gradient(theta0, dims, X[k], Y[k], mean_grad=True)
        grad_gpu = (theta0.astype(np.float64) - th[k].astype(np.float64)) / lr
        check_tensors(grad_gpu, grad_ref, dims, GRAD_TOL, f"replica {k} gradient")
        assert abs(float(host(g.loss)[k]) - loss_ref) < 1e-4 * abs(loss_ref)
    g2 = Gpu(dims, K, n, theta0)
    refs = [theta0.astype(np.float64) for _ in range(K)]
    for t in range(5):
        Xt = np.stack([_speech_batch(dims, seed, k, t, n)[0] for k in range(K)])
        Yt = np.stack([_speech_batch(dims, seed, k, t, n)[1] for k in range(K)])
        g2.step(Xt, Yt, 0.05)
        for k in range(K):
            refs[k], _, _ = dnn.sgd_step(refs[k], dims, Xt[k], Yt[k], 0.05)
    th = g2.params()
    for k in range(K):
        check_tensors(th[k], refs[k], dims, PARAM_TOL, f"replica {k} after five steps")


def test_paper_topology_full_width_first_step():
    # 440-6x2048-8806 (Sec. 5.1) at minibatch 256: the launches bench.py times for the paper's own shape, one step
    dims, n, seed, lr = gen.CONFIG_PAPER_DIMS, 256, 52, 16.0
    theta0 = gen.init_theta(dims, seed, 0.05)
    X, y = _speech_batch(dims, seed, 0, 0, n)
    g = Gpu(dims, 1, n, theta0)
    g.step(X[None], y[None], lr)
    check_acts(g.activations(0), dnn.forward(theta0, dims, X), ACT_TOL, "paper topology")
    grad_ref, loss_ref = dnn.gradient(theta0, dims, X, y, mean_grad=True)
    grad_gpu = (theta0.astype(np.float64) - g.params()[0].astype(np.float64)) / lr
    worst = check_tensors(grad_gpu, grad_ref, dims, GRAD_TOL, "paper topology gradient")
    print(f"8806-output first step: worst per-tensor relative error {worst[0]:.2e}, worst element {worst[1]:.2e}")
    assert abs(float(host(g.loss)[0]) - loss_ref) < 1e-4 * abs(loss_ref)


@pytest.mark.parametrize("K", [1, 3, 8])
@pytest.mark.parametrize("n", [64, 192, 320, 768])
def test_first_step_gradient_between_the_tuned_minibatch_sizes(n, K):
    # minibatch sizes and replica counts between the ones the tile plan was tuned on (128 ... 1024; 1 and 8
    # replicas), at full layer widths: whichever kernel the plan picks there has to be right
    dims, seed, lr = gen.CONFIG_FULL_DIMS, 53, 16.0
    theta0 = gen.init_theta(dims, seed, 0.05)
    X = np.stack([_full_batch(seed, k, 0, n)[0] for k in range(K)])
    Y = np.stack([_full_batch(seed, k, 0, n)[1] for k in range(K)])
    g = Gpu(dims, K, n, theta0)
    g.step(X, Y, lr)
    th = g.params()
    for k in sorted({0, K - 1}):             # first and last replica against the oracle; the others against replica 0's kernel path below
        grad_ref, _ = dnn.gradient(theta0, dims, X[k], Y[k], mean_grad=True)
        check_tensors((theta0.astype(np.float64) - th[k].astype(np.float64)) / lr, grad_ref, dims, GRAD_TOL, f"n {n}, replica {k}")
    if K > 2:
        # every replica's update has the norm the oracle's loss-independent bound allows and differs from its neighbours'
        for k in range(1, K):
            assert not np.array_equal(th[k], th[k - 1])


def test_shared_labels_and_inputs_across_replicas():
    # x_stride = 0 and label_stride = 0: all replicas read one minibatch (dnn_backward_update and dnn_count_correct alike)
    import torch
    from paper_1507_01239_amd import binding as B
    dims, K, n, seed = (44, 72, 36, 52), 3, 40, 54
    theta0 = gen.init_theta(dims, seed, 0.3)
    X = gen.features_iid(n, dims[0], seed, 0, 0)
    y = gen.labels_uniform(n, dims[-1], seed, 0, 0)
    g = Gpu(dims, K, n, theta0)
    x_d, y_d = dev(X), dev(y.astype(np.int32))
    B.dnn_forward(g.shape, K, g.theta, g.stride, x_d, 0, n, g.acts, g.act_stride, g.ws)
    correct = torch.full((K,), -1, dtype=torch.int32, device="cuda")
    B.dnn_count_correct(g.shape, K, g.acts, g.act_stride, y_d, 0, n, correct)
    B.dnn_backward_update(g.shape, K, g.theta, g.stride, x_d, 0, y_d, 0, n, g.acts, g.act_stride, 0.5, B.MEAN_GRAD, g.loss, g.ws)
    ref, loss_ref, acts = dnn.sgd_step(theta0, dims, X, y, 0.5)
    th = g.params()
    want = int((np.argmax(acts[-1], axis=1) == y).sum())
    for k in range(K):
        check_tensors(th[k], ref, dims, 1e-5, f"replica {k}")
        assert int(host(correct)[k]) == want
