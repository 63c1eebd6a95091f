"""ctypes binding of libmavg.so: the same names as include/mavg.h, argument marshalling only.

Device buffers are torch tensors (PyTorch is used for device memory and streams, nothing else) or raw
integer addresses.  Every call enqueues on torch's current stream unless `stream` is given.  There is
no CPU fallback: if the library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

# PyTorch provides the device memory and streams this library works on, and it ships its own copy of the
# HIP runtime.  It must be loaded BEFORE libmavg.so so that both use the same runtime instance: loading the
# library first pulls in the system runtime and torch's kernels then fault.
import torch  # noqa: F401  (import order matters)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmavg.so")

OK, E_NULL, E_DIM, E_ALIGN, E_FLAG, E_LAUNCH, E_WORKSPACE = 0, -1, -2, -3, -4, -5, -6
ACT_SIGMOID, ACT_TANH = 0, 1
MEAN_GRAD, USE_NGSGD, NG_FIRST, NG_APPLY_ONLY = 1, 2, 4, 8
VIS_BERNOULLI, VIS_GAUSSIAN = 0, 1
SAMPLE_V1 = 1
NG_APPLY, NG_UPDATE, NG_INIT_UPDATE = 0, 1, 2

_ERR = {E_NULL: "null pointer", E_DIM: "bad dimension or count", E_ALIGN: "bad alignment or stride",
        E_FLAG: "unknown flag or unsupported mode", E_LAUNCH: "HIP launch error", E_WORKSPACE: "workspace too small"}


class MavgError(RuntimeError):
    def __init__(self, code: int, where: str):
        detail = f": {lib.mavg_last_error().decode()}" if code == E_LAUNCH else ""
        super().__init__(f"{where}: error {code} ({_ERR.get(code, 'unknown')}{detail})")
        self.code = code


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_1507_01239_amd.build` "
                      "(or __graft_entry__.build()); there is no fallback path")
lib = C.CDLL(LIB_PATH)


class _Shape(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden_act", C.c_int32), ("dims", C.POINTER(C.c_int32))]


class Shape:
    """Network widths d_0..d_L and the hidden-unit nonlinearity (ACT_SIGMOID / ACT_TANH)."""

    def __init__(self, dims, hidden_act=0):
        self.dims = tuple(int(d) for d in dims)
        self.hidden_act = int(hidden_act)
        self._arr = (C.c_int32 * len(self.dims))(*self.dims)
        self._s = _Shape(len(self.dims) - 1, self.hidden_act, C.cast(self._arr, C.POINTER(C.c_int32)))

    @property
    def ref(self):
        return C.byref(self._s)


_p, _i32, _i64, _u32, _u64, _f = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_uint64, C.c_float
_SIG = {
    "mavg_version": (C.c_char_p, []),
    "mavg_last_error": (C.c_char_p, []),
    "mavg_param_count": (_i64, [_p]),
    "mavg_act_count": (_i64, [_p, _i32]),
    "mavg_workspace_bytes": (_i64, [_p, _i32, _i32, _u32, _i32]),
    "dnn_forward": (_i32, [_p, _i32, _p, _i64, _p, _i64, _i32, _p, _i64, _p, _i64, _p]),
    "dnn_backward_update": (_i32, [_p, _i32, _p, _i64, _p, _i64, _p, _i64, _i32, _p, _i64, _f, _u32,
                                   _p, _i64, _i32, _f, _f, _p, _p, _i64, _p]),
    "replicas_average": (_i32, [_p, _i64, _i64, _i32, _p]),
    "dnn_init_layer_from_rbm": (_i32, [_p, _i32, _p, _i64, _i32, _p, _p, _p]),
    "dnn_count_correct": (_i32, [_p, _i32, _p, _i64, _p, _i64, _i32, _p, _p]),
    "rbm_workspace_bytes": (_i64, [_i32, _i32, _i32]),
    "rbm_cd1_step": (_i32, [_i32, _i32, _i32, _p, _p, _p, _p, _p, _p, _p, _i32, _f, _f, _u64, _u32, _u32, _u32,
                            _p, _p, _i64, _p]),
    "rbm_cd1_step_static": (_i32, [_i32, _i32, _i32, _p, _p, _p, _p, _p, _p, _p, _i32, _f, _f, _u64, _u32, _u32, _u32,
                                   _p, _p]),
    "rbm_workspace_layout": (_i32, [_i32, _i32, _i32, _p]),
    "mavg_philox_fill": (_i32, [_p, _i64, _u32, _u64, _u32, _u32, _u32, _p]),
    "rbm_hidden_prob": (_i32, [_i32, _i32, _p, _p, _p, _i32, _p, _p, _i64, _p]),
    "ngsgd_state_bytes": (_i64, [_i32, _i32]),
    "ngsgd_workspace_bytes": (_i64, [_i32, _i32, _i32]),
    "ngsgd_state_init": (_i32, [_p, _i32, _i32, _p]),
    "ngsgd_precondition": (_i32, [_p, _i32, _i32, _p, _i64, _i32, _f, _f, _i32, _p, _i64, _p]),
    "mavg_gemm": (_i32, [_p, _i64, _i32, _p, _i64, _i32, _p, _i64, _i32, _i32, _i32, _i32, _p, _p, _i64, _f, _f,
                         _i32, _i32, _p, _i64, _p]),
    "mavg_gemm_workspace_bytes": (_i64, [_i32, _i32, _i32, _i32, _i32]),
    "mavg_gemm_grouped": (_i32, [_p, _i32, _i32, _i32, _p]),
}
EXPORTS = tuple(_SIG)
for _name, (_res, _args) in _SIG.items():
    _fn = getattr(lib, _name)
    _fn.restype, _fn.argtypes = _res, _args


def ptr(t):
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    if hasattr(t, "ctypes"):
        return t.ctypes.data
    raise TypeError(type(t))


def _nbytes(t):
    if t is None:
        return 0
    if hasattr(t, "element_size"):
        return t.numel() * t.element_size()
    return int(t.nbytes)


def _stream(stream):
    if stream is not None:
        return stream
    return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None


def _check(rc, where):
    if rc < 0:
        raise MavgError(int(rc), where)
    return rc


def mavg_version() -> str:
    return lib.mavg_version().decode()


def mavg_param_count(shape: Shape) -> int:
    return _check(lib.mavg_param_count(shape.ref), "mavg_param_count")


def mavg_act_count(shape: Shape, n: int) -> int:
    return _check(lib.mavg_act_count(shape.ref, n), "mavg_act_count")


def mavg_workspace_bytes(shape: Shape, n: int, k: int, flags: int = 0, ng_rank: int = 0) -> int:
    return _check(lib.mavg_workspace_bytes(shape.ref, n, k, flags, ng_rank), "mavg_workspace_bytes")


def dnn_forward(shape, k, theta, theta_stride, x, x_stride, n, acts, act_stride, workspace, stream=None,
                workspace_bytes=None):
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    return _check(lib.dnn_forward(shape.ref, k, ptr(theta), theta_stride, ptr(x), x_stride, n, ptr(acts), act_stride,
                                  ptr(workspace), wb, _stream(stream)), "dnn_forward")


def dnn_backward_update(shape, k, theta, theta_stride, x, x_stride, labels, label_stride, n, acts, act_stride, lr,
                        flags, loss_sum, workspace, ng_state=None, ng_state_stride=0, ng_rank=0, ng_alpha=4.0,
                        ng_eta=0.0, stream=None, workspace_bytes=None):
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    return _check(lib.dnn_backward_update(shape.ref, k, ptr(theta), theta_stride, ptr(x), x_stride, ptr(labels),
                                          label_stride, n, ptr(acts), act_stride, lr, flags, ptr(ng_state),
                                          ng_state_stride, ng_rank, ng_alpha, ng_eta, ptr(loss_sum), ptr(workspace), wb,
                                          _stream(stream)), "dnn_backward_update")


def replicas_average(theta, theta_stride, count, k, stream=None):
    return _check(lib.replicas_average(ptr(theta), theta_stride, count, k, _stream(stream)), "replicas_average")


def dnn_init_layer_from_rbm(shape, k, theta, theta_stride, layer, w, c, stream=None):
    return _check(lib.dnn_init_layer_from_rbm(shape.ref, k, ptr(theta), theta_stride, layer, ptr(w), ptr(c), _stream(stream)),
                  "dnn_init_layer_from_rbm")


def dnn_count_correct(shape, k, acts, act_stride, labels, label_stride, n, correct, stream=None):
    return _check(lib.dnn_count_correct(shape.ref, k, ptr(acts), act_stride, ptr(labels), label_stride, n, ptr(correct),
                                        _stream(stream)), "dnn_count_correct")


def rbm_workspace_bytes(n_vis, n_hid, n) -> int:
    return _check(lib.rbm_workspace_bytes(n_vis, n_hid, n), "rbm_workspace_bytes")


def rbm_cd1_step(n_vis, n_hid, vis_type, w, a, c, mw, ma, mc, v0, n, lr, momentum, seed, step, layer, flags,
                 recon_err, workspace, stream=None, workspace_bytes=None):
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    return _check(lib.rbm_cd1_step(n_vis, n_hid, vis_type, ptr(w), ptr(a), ptr(c), ptr(mw), ptr(ma), ptr(mc), ptr(v0), n,
                                   lr, momentum, seed, step, layer, flags, ptr(recon_err), ptr(workspace), wb,
                                   _stream(stream)), "rbm_cd1_step")


RBM_STATIC_SCRATCH_BYTES = 32 << 20


def rbm_cd1_step_static(n_vis, n_hid, vis_type, w, a, c, mw, ma, mc, v0, n, lr, momentum, seed, step, layer, flags,
                        recon_err, stream=None):
    return _check(lib.rbm_cd1_step_static(n_vis, n_hid, vis_type, ptr(w), ptr(a), ptr(c), ptr(mw), ptr(ma), ptr(mc),
                                          ptr(v0), n, lr, momentum, seed, step, layer, flags, ptr(recon_err),
                                          _stream(stream)), "rbm_cd1_step_static")


def rbm_workspace_layout(n_vis, n_hid, n):
    """((byte offset, row stride in floats) of P_h0, H0, V1, -P_h1) inside the 256-byte aligned workspace."""
    out = (C.c_int64 * 8)()
    _check(lib.rbm_workspace_layout(n_vis, n_hid, n, C.cast(out, C.c_void_p)), "rbm_workspace_layout")
    return tuple((int(out[2 * i]), int(out[2 * i + 1])) for i in range(4))


def mavg_philox_fill(out, nblocks, first_block, seed, step, layer, phase, stream=None):
    return _check(lib.mavg_philox_fill(ptr(out), nblocks, first_block, seed, step, layer, phase, _stream(stream)),
                  "mavg_philox_fill")


def rbm_hidden_prob(n_vis, n_hid, w, c, v, n, out, workspace, stream=None, workspace_bytes=None):
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    return _check(lib.rbm_hidden_prob(n_vis, n_hid, ptr(w), ptr(c), ptr(v), n, ptr(out), ptr(workspace), wb,
                                      _stream(stream)), "rbm_hidden_prob")


def ngsgd_state_bytes(dim, rank) -> int:
    return _check(lib.ngsgd_state_bytes(dim, rank), "ngsgd_state_bytes")


def ngsgd_workspace_bytes(dim, rank, n) -> int:
    return _check(lib.ngsgd_workspace_bytes(dim, rank, n), "ngsgd_workspace_bytes")


def ngsgd_state_init(state, dim, rank, stream=None):
    return _check(lib.ngsgd_state_init(ptr(state), dim, rank, _stream(stream)), "ngsgd_state_init")


def ngsgd_precondition(state, dim, rank, x, ldx, n, alpha, eta, update, workspace, stream=None, workspace_bytes=None):
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    return _check(lib.ngsgd_precondition(ptr(state), dim, rank, ptr(x), ldx, n, alpha, eta, update, ptr(workspace), wb,
                                         _stream(stream)), "ngsgd_precondition")


def mavg_gemm_workspace_bytes(m, n, k, cfg=-1, splits=0) -> int:
    return _check(lib.mavg_gemm_workspace_bytes(m, n, k, cfg, splits), "mavg_gemm_workspace_bytes")


def mavg_gemm(a, lda, a_kc, b, ldb, b_kc, c, ldc, m, n, k, epi, bias, aux, ldaux, alpha, beta, cfg, splits, workspace,
              stream=None, workspace_bytes=None):
    wb = _nbytes(workspace) if workspace_bytes is None else workspace_bytes
    return _check(lib.mavg_gemm(ptr(a), lda, int(a_kc), ptr(b), ldb, int(b_kc), ptr(c), ldc, m, n, k, epi, ptr(bias),
                                ptr(aux), ldaux, alpha, beta, cfg, splits, ptr(workspace), wb, _stream(stream)), "mavg_gemm")


class GemmProblem(C.Structure):
    """mavg_gemm_problem of include/mavg.h."""
    _fields_ = [("a", _p), ("lda", _i64), ("b", _p), ("ldb", _i64), ("c", _p), ("ldc", _i64),
                ("m", _i32), ("n", _i32), ("k", _i32), ("epi", _i32),
                ("bias", _p), ("aux", _p), ("ldaux", _i64), ("alpha", _f), ("beta", _f),
                ("rowsum_dst", _p), ("rowsum_alpha", _f), ("rowsum_beta", _f), ("a_pad4", _i32), ("b_pad4", _i32)]


def gemm_problem(a, lda, b, ldb, c, ldc, m, n, k, epi=0, bias=None, aux=None, ldaux=0, alpha=1.0, beta=0.0,
                 rowsum_dst=None, rowsum_alpha=1.0, rowsum_beta=0.0, a_pad4=False, b_pad4=False) -> GemmProblem:
    return GemmProblem(ptr(a), lda, ptr(b), ldb, ptr(c), ldc, m, n, k, epi, ptr(bias), ptr(aux), ldaux, alpha, beta,
                       ptr(rowsum_dst), rowsum_alpha, rowsum_beta, int(a_pad4), int(b_pad4))


def mavg_gemm_grouped(problems, a_kc, b_kc, stream=None):
    arr = (GemmProblem * len(problems))(*problems)
    return _check(lib.mavg_gemm_grouped(C.cast(arr, C.c_void_p), len(problems), int(a_kc), int(b_kc), _stream(stream)),
                  "mavg_gemm_grouped")
