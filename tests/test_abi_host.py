"""Host-side tests of the C ABI (no GPU): the library loads, exports every symbol the header declares,
sizes are right, and invalid arguments are rejected before anything is launched."""
import os
import re

import numpy as np
import pytest

import gen
from paper_1507_01239_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    src = open(os.path.join(ROOT, "include", "mavg.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(?:int32_t|int64_t|const char\*)\s+(\w+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert {"dnn_forward", "dnn_backward_update", "replicas_average", "rbm_cd1_step", "ngsgd_precondition"} <= set(names)
    for n in names:
        assert hasattr(B.lib, n), n
    assert set(names) == set(B.EXPORTS)
    assert "gfx950" in B.mavg_version()


def test_sizes_match_fixture_and_generator():
    for line in open(os.path.join(ROOT, "tests", "golden", "topology_param_count.txt")):
        if line.startswith("#") or not line.strip():
            continue
        lhs, rhs = line.split("->")
        dims = tuple(int(t) for t in lhs.split())
        s = B.Shape(dims)
        assert B.mavg_param_count(s) == int(rhs) == gen.param_count(dims)
        assert B.mavg_act_count(s, 7) == 7 * sum(dims[1:])
    s = B.Shape(gen.CONFIG_FULL_DIMS)
    assert B.mavg_workspace_bytes(s, 256, 1, B.MEAN_GRAD) > 2 * 256 * 8000 * 4
    assert B.mavg_workspace_bytes(s, 256, 8, B.MEAN_GRAD) >= B.mavg_workspace_bytes(s, 256, 1, B.MEAN_GRAD)


def _rc(fn, *a, **k):
    try:
        fn(*a, **k)
    except B.MavgError as e:
        return e.code
    return 0


def test_bad_shapes_are_rejected():
    assert B.lib.mavg_param_count(None) == B.E_NULL
    assert _rc(B.mavg_param_count, B.Shape((4,))) == B.E_DIM            # zero layers
    assert _rc(B.mavg_param_count, B.Shape((4, 0, 3))) == B.E_DIM
    assert _rc(B.mavg_act_count, B.Shape((4, 3)), 0) == B.E_DIM
    assert _rc(B.mavg_workspace_bytes, B.Shape((4, 3)), 8, 0) == B.E_DIM
    assert _rc(B.mavg_workspace_bytes, B.Shape((4, 3)), 8, 1, 16) == B.E_FLAG
    assert _rc(B.mavg_workspace_bytes, B.Shape((4, 3)), 8, 1, B.USE_NGSGD | B.NG_FIRST | B.NG_APPLY_ONLY, 2) == B.E_FLAG
    assert _rc(B.mavg_param_count, B.Shape(tuple([3] * 70))) == B.E_DIM  # too many layers
    assert _rc(B.mavg_param_count, B.Shape((4, 3), hidden_act=7)) == B.E_FLAG      # unknown nonlinearity
    assert B.mavg_param_count(B.Shape((4, 3), hidden_act=B.ACT_TANH)) == 15


def test_dnn_calls_validate_before_touching_the_device():
    s = B.Shape((8, 4, 4))
    A = 1 << 20     # a fake, aligned, never dereferenced address
    big = 1 << 30
    ok = dict(workspace=A, workspace_bytes=big, stream=0)
    assert _rc(B.dnn_forward, s, 1, None, 0, A, 0, 4, A, 0, **ok) == B.E_NULL
    assert _rc(B.dnn_forward, s, 0, A, 0, A, 0, 4, A, 0, **ok) == B.E_DIM
    assert _rc(B.dnn_forward, s, 1, A, 0, A, 0, 0, A, 0, **ok) == B.E_DIM
    assert _rc(B.dnn_forward, s, 1, A + 4, 0, A, 0, 4, A, 0, **ok) == B.E_ALIGN
    assert _rc(B.dnn_forward, s, 2, A, 10, A, 0, 4, A, 64, **ok) == B.E_ALIGN        # stride < P
    assert _rc(B.dnn_forward, s, 2, A, 64, A, 0, 4, A, 8, **ok) == B.E_ALIGN         # act stride too small
    bw = lambda **kw: _rc(B.dnn_backward_update, s, kw.get("k", 1), kw.get("theta", A), 64, A, 0, kw.get("labels", A), 0,
                          kw.get("n", 4), A, 64, 0.1, kw.get("flags", 1), None, kw.get("ws", A),
                          workspace_bytes=kw.get("wb", big), stream=0,
                          ng_state=kw.get("ng", None), ng_rank=kw.get("rank", 0), ng_state_stride=kw.get("ngs", 0),
                          ng_eta=0.1)
    assert bw(labels=None) == B.E_NULL
    assert bw(flags=16) == B.E_FLAG
    assert bw(flags=B.USE_NGSGD | B.NG_FIRST | B.NG_APPLY_ONLY) == B.E_FLAG     # the first minibatch always folds
    assert bw(ws=None) == B.E_WORKSPACE
    assert bw(wb=16) == B.E_WORKSPACE
    assert bw(flags=3) == B.E_NULL                      # NG-SGD without a state
    assert bw(flags=3, ng=A, rank=0) == B.E_DIM
    assert bw(flags=3, ng=A, rank=4) == B.E_DIM         # rank must be < every factor dimension
    assert bw(n=-1) == B.E_DIM
    assert bw(n=65535) == B.E_DIM                       # rows (+ 1 for the loss) are a grid dimension
    assert _rc(B.dnn_forward, s, 1, A, 0, A, 0, 65535, A, 0, **ok) == B.E_DIM


def test_replicas_average_validation():
    A = 1 << 20
    assert _rc(B.replicas_average, None, 8, 8, 2, stream=0) == B.E_NULL
    assert _rc(B.replicas_average, A, 8, -1, 2, stream=0) == B.E_DIM
    assert _rc(B.replicas_average, A, 8, 8, 0, stream=0) == B.E_DIM
    assert _rc(B.replicas_average, A, 8, 8, 65, stream=0) == B.E_DIM
    assert _rc(B.replicas_average, A + 8, 8, 8, 2, stream=0) == B.E_ALIGN
    assert _rc(B.replicas_average, A, 4, 8, 2, stream=0) == B.E_ALIGN     # stride < count
    assert _rc(B.replicas_average, A, 10, 8, 2, stream=0) == B.E_ALIGN    # stride not a multiple of 4
    assert _rc(B.replicas_average, A, 8, 0, 2, stream=0) == 0             # empty: no-op, nothing launched


def test_rbm_and_gemm_validation():
    A = 1 << 20
    big = 1 << 30
    call = lambda **kw: _rc(B.rbm_cd1_step, kw.get("V", 8), kw.get("H", 4), kw.get("vt", 0), kw.get("w", A), A, A, A, A, A, A,
                            kw.get("n", 4), 0.1, 0.9, 1, 0, 0, kw.get("flags", 0), None, kw.get("ws", A),
                            workspace_bytes=kw.get("wb", big), stream=0)
    assert call(w=None) == B.E_NULL
    assert call(V=0) == B.E_DIM
    assert call(vt=2) == B.E_FLAG
    assert call(flags=2) == B.E_FLAG
    assert call(vt=1, flags=1) == B.E_FLAG              # cannot Bernoulli-sample Gaussian visibles
    assert call(w=A + 4) == B.E_ALIGN
    assert call(wb=8) == B.E_WORKSPACE
    assert B.rbm_workspace_bytes(440, 2048, 256) > 3 * 256 * 2048 * 4
    assert _rc(B.rbm_workspace_bytes, 0, 4, 4) == B.E_DIM
    g = lambda **kw: _rc(B.mavg_gemm, kw.get("a", A), kw.get("lda", 64), 1, A, 64, 1, A, 16, 8, 8, 64, kw.get("epi", 0),
                         kw.get("bias", None), None, 0, 1.0, 0.0, kw.get("cfg", -1), kw.get("splits", 0), A,
                         workspace_bytes=kw.get("wb", big), stream=0)
    assert g(a=None) == B.E_NULL
    assert g(lda=4) == B.E_ALIGN
    assert g(epi=9) == B.E_FLAG
    assert g(epi=1) == B.E_NULL                          # bias epilogue without a bias
    assert g(cfg=99) == B.E_FLAG
    assert g(splits=2, wb=0) == B.E_WORKSPACE
    pr = lambda **kw: B.gemm_problem(kw.get("a", A), kw.get("lda", 64), A, 64, A, 64, 8, 8, 16, epi=kw.get("epi", 0))
    gg = lambda probs, a_kc=1: _rc(B.mavg_gemm_grouped, probs, a_kc, 1, stream=0)
    assert B.lib.mavg_gemm_grouped(None, 1, 1, 1, None) == B.E_NULL
    assert gg([pr()] * 9) == B.E_DIM                     # at most 8 problems per launch
    assert gg([pr(a=None)]) == B.E_NULL
    assert gg([pr(lda=4)]) == B.E_ALIGN
    assert gg([pr(epi=7)]) == B.E_FLAG
    assert gg([pr(epi=1)]) == B.E_NULL                   # bias epilogue without a bias
