"""GPU parity of the steps before and after the hot path: the greedy RBM stack and the DNN initialised from it
(Sec. 5.1, 5.3), the held-out frame accuracy and the schedules it drives (Sec. 5.6), against the oracle.

The stack is not teacher-forced (the single CD-1 step is, in test_gpu_rbm.py): a handful of updates per RBM
from the same start, then the parameters are compared within 1e-3 (the bar for parameters after many steps).
A Bernoulli decision that falls on the other side in float32 would move single entries of the statistics by
lr/n; none occurred at these sizes and seeds, and the tolerance would not hide a systematic error."""
import numpy as np
import pytest

import gen
from oracle import dnn as odnn
from oracle import pretrain as opre
from oracle import schedule as osch
from tests.util import dev, host, rel_err, workspace

pytestmark = pytest.mark.gpu


def _stack_case(widths, n, nmb, seed):
    mbs = [gen.features_speech_like(n, widths[0], seed, 0, t).astype(np.float32) for t in range(nmb)]
    init = [tuple(t.astype(np.float32) for t in gen.rbm_params(widths[l - 1], widths[l], seed, l)) for l in range(1, len(widths))]
    return mbs, init


@pytest.mark.parametrize("widths,n,steps", [([40, 64, 48, 33], 32, 6), ([440, 256, 192], 96, 3)])
def test_stack_and_initialisation_match_the_oracle(widths, n, steps):
    import torch
    from paper_1507_01239_amd import binding as B
    from paper_1507_01239_amd import pretrain as P
    seed = 77
    mbs, init = _stack_case(widths, n, 3, seed)
    ref_stack, ref_errs = opre.pretrain_stack(widths, mbs, init, steps, 0.01, 0.4, 0.9, seed)
    d_init = [tuple(dev(t) for t in rbm) for rbm in init]
    errs = P.pretrain_stack(widths, [dev(m) for m in mbs], d_init, steps, 0.01, 0.4, 0.9, seed)
    torch.cuda.synchronize()
    for l, (rbm_g, rbm_o) in enumerate(zip(d_init, ref_stack), start=1):
        for name, g, o in zip("Wac", rbm_g, rbm_o):
            assert rel_err(host(g), o) < 1e-3, (l, name)
        assert rel_err(host(errs[l - 1]), np.array(ref_errs[l - 1])) < 1e-3

    # initialise 3 replicas of a DNN with one more (softmax) layer from the GPU's stack
    dims = widths + [29]
    k = 3
    shape = B.Shape(dims)
    Pn = B.mavg_param_count(shape)
    stride = (Pn + 63) // 64 * 64
    theta0 = np.stack([gen.init_theta(dims, seed + r, 0.1) for r in range(k)]).astype(np.float32)
    theta = torch.zeros(k, stride, device="cuda")
    theta[:, :Pn] = dev(theta0)
    P.init_dnn_from_stack(shape, k, theta, stride, d_init)
    torch.cuda.synchronize()
    for r in range(k):
        want = opre.init_dnn_from_stack(theta0[r], dims, [tuple(host(t) for t in rbm) for rbm in d_init])
        assert np.array_equal(host(theta[r, :Pn]), want.astype(np.float32))      # a copy: bit for bit
    assert np.all(host(theta[:, Pn:]) == 0)                                      # padding between replicas untouched


def test_init_layer_rejects_bad_arguments():
    import torch
    from paper_1507_01239_amd import binding as B
    shape = B.Shape([8, 6, 4])
    th, w, c = torch.zeros(100, device="cuda"), torch.zeros(6, 8, device="cuda"), torch.zeros(6, device="cuda")
    for layer in (0, 3):
        with pytest.raises(B.MavgError) as e:
            B.dnn_init_layer_from_rbm(shape, 1, th, 0, layer, w, c)
        assert e.value.args[0].find(str(B.E_DIM)) >= 0
    with pytest.raises(B.MavgError):
        B.dnn_init_layer_from_rbm(shape, 1, th, 0, 1, None, c)
    with pytest.raises(B.MavgError):
        B.dnn_init_layer_from_rbm(shape, 2, th, 10, 1, w, c)       # replica stride shorter than the parameter vector


@pytest.mark.parametrize("dims,n,k", [([40, 64, 64, 32], 96, 3), ([440, 128, 8000], 64, 1), ([20, 16, 3], 5, 2)])
def test_frame_accuracy_matches_the_oracle(dims, n, k):
    import torch
    from paper_1507_01239_amd import binding as B
    from paper_1507_01239_amd import schedule as S
    seed = 5
    shape = B.Shape(dims)
    Pn = B.mavg_param_count(shape)
    theta0 = np.stack([gen.init_theta(dims, seed + r, 0.3) for r in range(k)]).astype(np.float32)
    X = np.stack([gen.features_iid(n, dims[0], seed, r, 0) for r in range(k)]).astype(np.float32)
    # labels: the oracle's own arg max on two thirds of the rows (so that hits are plentiful), random elsewhere
    post = [odnn.forward(theta0[r], dims, X[r])[-1] for r in range(k)]
    rng = np.random.default_rng(seed)
    y = np.stack([np.where(rng.random(n) < 0.66, np.argmax(post[r], axis=1), rng.integers(0, dims[-1], n)) for r in range(k)]).astype(np.int32)
    stride = (Pn + 63) // 64 * 64
    theta = torch.zeros(k, stride, device="cuda")
    theta[:, :Pn] = dev(theta0)
    x, yd = dev(X), dev(y)
    astride = (B.mavg_act_count(shape, n) + 63) // 64 * 64
    acts = torch.empty(k, astride, device="cuda")
    ws = workspace(B.mavg_workspace_bytes(shape, n, k, 0))
    got = S.frame_accuracy(shape, k, theta, stride, x, n * dims[0], yd, n, n, acts, astride, ws)
    for r in range(k):
        p = post[r]
        top2 = np.sort(p, axis=1)[:, -2:]
        clear = (top2[:, 1] - top2[:, 0]) > 1e-5 * top2[:, 1]        # rows whose arg max is decided beyond float32 noise
        hits_clear = int(((np.argmax(p, axis=1) == y[r]) & clear).sum())
        n_unclear = int((~clear).sum())
        got_hits = round(got[r] * n)
        assert hits_clear <= got_hits <= hits_clear + n_unclear
        if n_unclear == 0:
            assert got[r] == osch.frame_accuracy(p, y[r])
    # a second call overwrites the counts instead of adding to them
    again = S.frame_accuracy(shape, k, theta, stride, x, n * dims[0], yd, n, n, acts, astride, ws)
    assert again == got


def test_arg_max_takes_the_lowest_index_among_equal_posteriors():
    import torch
    from paper_1507_01239_amd import binding as B
    dims = [4, 3, 600]
    shape = B.Shape(dims)
    n = 4
    acts = torch.zeros(B.mavg_act_count(shape, n), device="cuda")
    post = acts[n * 3:].view(n, 600)
    post[0, 599] = 0.5; post[0, 300] = 0.5       # tie: 300 wins
    post[1, 0] = 0.2; post[1, 1] = 0.2           # tie at the very start: 0 wins
    post[2, 257] = 0.9                           # single maximum in the second sweep of the row
    # row 3: all equal (zeros): class 0 wins
    for labels, want in (([300, 0, 257, 0], 4), ([599, 1, 257, 5], 1)):
        correct = torch.full((1,), 123, dtype=torch.int32, device="cuda")
        B.dnn_count_correct(shape, 1, acts, 0, dev(np.array(labels, np.int32)), 0, n, correct)
        assert int(correct.item()) == want


def test_full_width_stack_of_six_rbms_and_initialisation():
    # Sec. 5.1 at size: 440 -> 2048 and five RBMs of 2048 -> 2048, minibatch 256, two CD-1 updates per RBM from the
    # same start on both sides (a longer run is a free-running comparison: see the 500-minibatch test of the single
    # RBMs), then the copy into the six hidden layers of the 440-6x2048-8000 network
    import torch
    from paper_1507_01239_amd import binding as B
    from paper_1507_01239_amd import pretrain as P
    seed, n, steps = 78, 256, 2
    widths = list(gen.CONFIG_FULL_DIMS[:-1])
    mbs, init = _stack_case(widths, n, 2, seed)
    ref_stack, ref_errs = opre.pretrain_stack(widths, mbs, init, steps, 0.01, 0.4, 0.9, seed)
    d_init = [tuple(dev(t) for t in r) for r in init]
    errs = P.pretrain_stack(widths, [dev(m) for m in mbs], d_init, steps, 0.01, 0.4, 0.9, seed)
    torch.cuda.synchronize()
    for l, (rbm_g, rbm_o) in enumerate(zip(d_init, ref_stack), start=1):
        for name, g, o in zip("Wac", rbm_g, rbm_o):
            assert rel_err(host(g), o) < 1e-3, (l, name)
        assert rel_err(host(errs[l - 1]), np.array(ref_errs[l - 1])) < 1e-3, l
    dims = gen.CONFIG_FULL_DIMS
    shape = B.Shape(dims)
    Pn = B.mavg_param_count(shape)
    theta0 = gen.init_theta(dims, seed, 0.05)
    theta = dev(theta0)
    P.init_dnn_from_stack(shape, 1, theta, Pn, d_init)
    torch.cuda.synchronize()
    want = opre.init_dnn_from_stack(theta0, dims, [tuple(host(t) for t in r) for r in d_init])
    assert np.array_equal(host(theta), want.astype(np.float32))
