// dnn_forward / dnn_backward_update: host-side validation and the sequence of kernel launches for
// one minibatch of k replicas (the replica index is the batch dimension of every launch).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mavg.h"
#include "gemm.h"
#include "kernels.h"
#include "ng_internal.h"

using namespace mavg;

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

int check_shape(const mavg_shape* sh) {
    if (!sh || !sh->dims) return MAVG_E_NULL;
    if (sh->n_layers < 1 || sh->n_layers > MAVG_MAX_LAYERS) return MAVG_E_DIM;
    if (sh->hidden_act != MAVG_ACT_SIGMOID && sh->hidden_act != MAVG_ACT_TANH) return MAVG_E_FLAG;
    for (int l = 0; l <= sh->n_layers; ++l)
        if (sh->dims[l] < 1) return MAVG_E_DIM;
    return MAVG_OK;
}

// offsets (in floats) of W_l and b_l inside theta, and of A_l inside acts, l = 1..L
struct Layout {
    int L;
    int d[MAVG_MAX_LAYERS + 1];
    int64_t w_off[MAVG_MAX_LAYERS + 1], b_off[MAVG_MAX_LAYERS + 1], a_off[MAVG_MAX_LAYERS + 1];
    int64_t P, acts;
    int dmax;      // widest layer output
};

Layout make_layout(const mavg_shape* sh, int n) {
    Layout y;
    y.L = sh->n_layers;
    int64_t off = 0, aoff = 0;
    y.dmax = 0;
    y.d[0] = sh->dims[0];
    for (int l = 1; l <= y.L; ++l) {
        y.d[l] = sh->dims[l];
        y.w_off[l] = off;
        off += (int64_t)sh->dims[l] * sh->dims[l - 1];
        y.b_off[l] = off;
        off += sh->dims[l];
        y.a_off[l] = aoff;
        aoff += (int64_t)n * sh->dims[l];
        if (sh->dims[l] > y.dmax) y.dmax = sh->dims[l];
    }
    y.P = off;
    y.acts = aoff;
    return y;
}

// Workspace carve-up shared by forward and backward.
struct Workspace {
    int64_t ld_delta[MAVG_MAX_LAYERS + 1];    // row stride of delta_l (d_l rounded up to a multiple of 4)
    int64_t off_delta[MAVG_MAX_LAYERS + 1];   // delta_l for every layer: all are alive until the grouped weight update
    int64_t off_rowloss, off_gemm, gemm_floats;
    int64_t off_ng, ng_floats;                // NG-SGD: preconditioned copies + its own scratch
    int64_t total_floats;
};

Workspace make_workspace(const Layout& y, int n, int k, uint32_t flags, int ng_rank) {
    Workspace w;
    int64_t g = 0;
    for (int l = 1; l <= y.L; ++l) {
        int64_t f = gemm_ws_floats(n, y.d[l], y.d[l - 1], k);                  // forward
        if (f > g) g = f;
        if (l > 1) { f = gemm_ws_floats(n, y.d[l - 1], y.d[l], k); if (f > g) g = f; }   // back-propagation
        f = gemm_ws_floats(y.d[l], y.d[l - 1] + 1, n, k);                      // weight + bias gradient (NG-SGD path)
        if (f > g) g = f;
    }
    w.gemm_floats = round_up(g, 64);
    int64_t off = 0;
    for (int l = 1; l <= y.L; ++l) {
        w.ld_delta[l] = round_up(y.d[l], 4);
        w.off_delta[l] = off;
        off += round_up((int64_t)k * n * w.ld_delta[l], 64);
    }
    w.off_rowloss = off;  off += round_up((int64_t)k * n, 64);
    w.off_gemm = off;     off += w.gemm_floats;
    w.off_ng = off;
    w.ng_floats = (flags & MAVG_USE_NGSGD) ? ng_dnn_ws_floats(y.d, y.L, n, k, ng_rank) : 0;
    off += w.ng_floats;
    w.total_floats = off;
    return w;
}

}  // namespace

extern "C" const char* mavg_version(void) { return "mavg 0.1 (gfx950, fp32 MFMA)"; }

extern "C" int64_t mavg_param_count(const mavg_shape* shape) {
    const int rc = check_shape(shape);
    if (rc) return rc;
    return make_layout(shape, 1).P;
}

extern "C" int64_t mavg_act_count(const mavg_shape* shape, int32_t n) {
    const int rc = check_shape(shape);
    if (rc) return rc;
    if (n < 1) return MAVG_E_DIM;
    return make_layout(shape, n).acts;
}

extern "C" int64_t mavg_workspace_bytes(const mavg_shape* shape, int32_t n, int32_t k, uint32_t flags, int32_t ng_rank) {
    const int rc = check_shape(shape);
    if (rc) return rc;
    if (n < 1 || k < 1) return MAVG_E_DIM;
    if (flags & ~(MAVG_MEAN_GRAD | MAVG_USE_NGSGD | MAVG_NG_FIRST | MAVG_NG_APPLY_ONLY)) return MAVG_E_FLAG;
    if ((flags & MAVG_NG_FIRST) && (flags & MAVG_NG_APPLY_ONLY)) return MAVG_E_FLAG;
    if ((flags & MAVG_USE_NGSGD) && (ng_rank < 1 || ng_rank > 64)) return MAVG_E_DIM;
    const Layout y = make_layout(shape, n);
    return make_workspace(y, n, k, flags, ng_rank).total_floats * 4 + 256;
}

static int check_common(const mavg_shape* shape, int32_t k, const void* theta, int64_t theta_stride, const void* x,
                        int64_t x_stride, int32_t n, const void* acts, int64_t act_stride, Layout* out) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!theta || !x || !acts) return MAVG_E_NULL;
    if (k < 1 || n < 1) return MAVG_E_DIM;
    if (k > 65535 || n > 65534) return MAVG_E_DIM;      // replicas and rows (+ 1 for the loss) are grid dimensions of some launches
    *out = make_layout(shape, n);
    if (!aligned16(theta) || !aligned16(x) || !aligned16(acts)) return MAVG_E_ALIGN;
    if (k > 1) {
        if (theta_stride < out->P || (theta_stride & 3)) return MAVG_E_ALIGN;
        if (x_stride != 0 && (x_stride < (int64_t)n * out->d[0] || (x_stride & 3))) return MAVG_E_ALIGN;
        if (act_stride < out->acts || (act_stride & 3)) return MAVG_E_ALIGN;
    }
    return MAVG_OK;
}

static float* ws_base(void* workspace) {
    return reinterpret_cast<float*>((reinterpret_cast<uintptr_t>(workspace) + 255u) & ~uintptr_t(255));
}

extern "C" int32_t dnn_forward(const mavg_shape* shape, int32_t k, const float* theta, int64_t theta_stride,
                               const float* x, int64_t x_stride, int32_t n, float* acts, int64_t act_stride,
                               void* workspace, int64_t workspace_bytes, void* stream) {
    Layout y;
    int rc = check_common(shape, k, theta, theta_stride, x, x_stride, n, acts, act_stride, &y);
    if (rc) return rc;
    const Workspace w = make_workspace(y, n, k, 0, 0);
    if (w.total_floats > 0 && (!workspace || workspace_bytes < w.total_floats * 4 + 256)) return MAVG_E_WORKSPACE;
    float* ws = workspace ? ws_base(workspace) : nullptr;
    hipStream_t s = static_cast<hipStream_t>(stream);
    for (int l = 1; l <= y.L; ++l) {
        GemmDesc g;
        g.M = n; g.N = y.d[l]; g.K = y.d[l - 1]; g.batch = k;
        if (l == 1) { g.A = x; g.lda = y.d[0]; g.a_bstride = x_stride; }
        else { g.A = acts + y.a_off[l - 1]; g.lda = y.d[l - 1]; g.a_bstride = act_stride; }
        g.a_kc = true;
        g.B = theta + y.w_off[l]; g.ldb = y.d[l - 1]; g.b_bstride = theta_stride; g.b_kc = true;
        g.C = acts + y.a_off[l]; g.ldc = y.d[l]; g.c_bstride = act_stride;
        g.epi.kind = (l < y.L) ? EPI_BIAS_SIGMOID : EPI_BIAS;
        g.epi.act_tanh = shape->hidden_act == MAVG_ACT_TANH;
        g.epi.bias = theta + y.b_off[l]; g.epi.bias_bstride = theta_stride;
        if (gemm_launch(g, ws ? ws + w.off_gemm : nullptr, w.gemm_floats, s) != 0) return MAVG_E_LAUNCH;
    }
    if (softmax_rows_launch(acts + y.a_off[y.L], y.d[y.L], act_stride, n, y.d[y.L], k, s) != 0) return MAVG_E_LAUNCH;
    return MAVG_OK;
}

extern "C" int32_t dnn_backward_update(const mavg_shape* shape, int32_t k, float* theta, int64_t theta_stride,
                                       const float* x, int64_t x_stride, const int32_t* labels, int64_t label_stride,
                                       int32_t n, const float* acts, int64_t act_stride, float lr, uint32_t flags,
                                       void* ng_state, int64_t ng_state_stride, int32_t ng_rank, float ng_alpha,
                                       float ng_eta, float* loss_sum, void* workspace, int64_t workspace_bytes,
                                       void* stream) {
    Layout y;
    int rc = check_common(shape, k, theta, theta_stride, x, x_stride, n, acts, act_stride, &y);
    if (rc) return rc;
    if (!labels) return MAVG_E_NULL;
    if (flags & ~(MAVG_MEAN_GRAD | MAVG_USE_NGSGD | MAVG_NG_FIRST | MAVG_NG_APPLY_ONLY)) return MAVG_E_FLAG;
    if ((flags & MAVG_NG_FIRST) && (flags & MAVG_NG_APPLY_ONLY)) return MAVG_E_FLAG;
    if (k > 1 && label_stride != 0 && label_stride < n) return MAVG_E_ALIGN;
    const bool ng = (flags & MAVG_USE_NGSGD) != 0;
    if (ng) {
        if (!ng_state) return MAVG_E_NULL;
        if (ng_rank < 1 || ng_rank > 64) return MAVG_E_DIM;
        for (int l = 1; l <= y.L; ++l)
            if (ng_rank >= y.d[l] || ng_rank >= y.d[l - 1] + 1) return MAVG_E_DIM;
        int dm = y.d[0];
        for (int l = 1; l <= y.L; ++l) if (y.d[l] > dm) dm = y.d[l];
        if (!aligned16(ng_state) || (ng_state_stride & 15) || ng_state_stride < ngsgd_state_bytes(dm + 1, ng_rank)) return MAVG_E_ALIGN;
        if (!(ng_alpha > 0.f) || !(ng_eta > 0.f && ng_eta < 1.f)) return MAVG_E_DIM;
    }
    const Workspace w = make_workspace(y, n, k, flags, ng_rank);
    if (!workspace || workspace_bytes < w.total_floats * 4 + 256) return MAVG_E_WORKSPACE;
    if (!aligned16(labels) || (loss_sum && (reinterpret_cast<uintptr_t>(loss_sum) & 3u))) return MAVG_E_ALIGN;
    float* ws = ws_base(workspace);
    hipStream_t s = static_cast<hipStream_t>(stream);
    float* gws = ws + w.off_gemm;
    const float scale = (flags & MAVG_MEAN_GRAD) ? 1.0f / (float)n : 1.0f;
    auto delta_of = [&](int l) { return ws + w.off_delta[l]; };
    auto dstride_of = [&](int l) { return (int64_t)n * w.ld_delta[l]; };

    if (ce_delta_launch(acts + y.a_off[y.L], y.d[y.L], act_stride, labels, label_stride, delta_of(y.L), w.ld_delta[y.L],
                        dstride_of(y.L), loss_sum, n, y.d[y.L], k, scale, s) != 0) return MAVG_E_LAUNCH;

    // 1. the chain: delta_{l-1} = (delta_l W_l) * A_{l-1} (1 - A_{l-1}), l = L..2, with every W_l as it was in the
    //    forward pass (no weight is touched before the chain is complete)
    for (int l = y.L; l >= 2; --l) {
        GemmDesc g;
        g.M = n; g.N = y.d[l - 1]; g.K = y.d[l]; g.batch = k;
        g.A = delta_of(l); g.lda = w.ld_delta[l]; g.a_bstride = dstride_of(l); g.a_kc = true;
        g.B = theta + y.w_off[l]; g.ldb = y.d[l - 1]; g.b_bstride = theta_stride; g.b_kc = false;
        g.C = delta_of(l - 1); g.ldc = w.ld_delta[l - 1]; g.c_bstride = dstride_of(l - 1);
        g.epi.kind = EPI_MUL_DSIGMOID;
        g.epi.act_tanh = shape->hidden_act == MAVG_ACT_TANH;
        g.epi.aux = acts + y.a_off[l - 1]; g.epi.ldaux = y.d[l - 1]; g.epi.aux_bstride = act_stride;
        if (gemm_launch(g, gws, w.gemm_floats, s) != 0) return MAVG_E_LAUNCH;
    }
    // 2. the updates.  Plain SGD: W_l <- W_l - lr delta_l^T A_{l-1} for all layers in ONE grouped launch, with
    //    b_l <- b_l - lr colsum(delta_l) fused as the row sums of each GEMM's A operand (delta_l^T).
    if (!ng) {
        GemmDesc g[MAVG_MAX_LAYERS];
        for (int l = 1; l <= y.L; ++l) {
            GemmDesc& q = g[l - 1];
            q.M = y.d[l]; q.N = y.d[l - 1]; q.K = n; q.batch = k;
            q.A = delta_of(l); q.lda = w.ld_delta[l]; q.a_bstride = dstride_of(l); q.a_kc = false;
            q.a_pad4 = true;       // rows of delta_l are ld_delta = round_up(d_l, 4) floats long
            q.B = (l == 1) ? x : acts + y.a_off[l - 1]; q.ldb = y.d[l - 1]; q.b_bstride = (l == 1) ? x_stride : act_stride;
            q.b_kc = false;
            q.C = theta + y.w_off[l]; q.ldc = y.d[l - 1]; q.c_bstride = theta_stride;
            q.epi.kind = EPI_AXPBY; q.epi.alpha = -lr; q.epi.beta = 1.f;
            q.epi.rowsum_dst = theta + y.b_off[l]; q.epi.rowsum_bstride = theta_stride;
            q.epi.rowsum_alpha = -lr; q.epi.rowsum_beta = 1.f;
        }
        if (gemm_launch_grouped(g, y.L, s) != 0) return MAVG_E_LAUNCH;
    } else {
        // the first minibatch (three folds from the initial state first) layer by layer; afterwards every layer
        // side in the same launches
        static thread_local NgLayerArgs la[MAVG_MAX_LAYERS];
        for (int l = y.L; l >= 1; --l) {
            NgLayerArgs& a = la[l - 1];
            a.dims = y.d; a.L = y.L; a.l = l;
            a.k = k; a.n = n; a.d_in = y.d[l - 1]; a.d_out = y.d[l];
            a.A_in = (l == 1) ? x : acts + y.a_off[l - 1]; a.a_ld = y.d[l - 1]; a.a_bstride = (l == 1) ? x_stride : act_stride;
            a.delta = delta_of(l); a.ldd = w.ld_delta[l]; a.d_bstride = dstride_of(l);
            a.W = theta + y.w_off[l]; a.b = theta + y.b_off[l]; a.theta_stride = theta_stride;
            a.state_in = static_cast<char*>(ng_state) + (int64_t)(2 * (l - 1)) * ng_state_stride;
            a.state_out = static_cast<char*>(ng_state) + (int64_t)(2 * (l - 1) + 1) * ng_state_stride;
            a.state_rstride = (int64_t)2 * y.L * ng_state_stride;
            a.rank = ng_rank; a.alpha = ng_alpha; a.eta = ng_eta; a.lr = lr;
            a.mode = (flags & MAVG_NG_FIRST) ? 2 : (flags & MAVG_NG_APPLY_ONLY) ? 0 : 1;
            a.ws = ws + w.off_ng; a.ws_floats = w.ng_floats;
            a.gemm_ws = gws; a.gemm_ws_floats = w.gemm_floats;
            if ((flags & MAVG_NG_FIRST) && ng_layer_update(a, s) != 0) return MAVG_E_LAUNCH;
        }
        if (!(flags & MAVG_NG_FIRST)) {
            if (ng_dnn_update(la, y.L, static_cast<char*>(ng_state), ng_state_stride, s) != 0) return MAVG_E_LAUNCH;
        } else if (ng_dnn_finish(y.d, y.L, n, k, ng_rank, ng_eta, static_cast<char*>(ng_state), ng_state_stride, ws + w.off_ng, s) != 0) {
            return MAVG_E_LAUNCH;
        }
    }
    return MAVG_OK;
}

extern "C" int32_t dnn_init_layer_from_rbm(const mavg_shape* shape, int32_t k, float* theta, int64_t theta_stride,
                                           int32_t layer, const float* w, const float* c, void* stream) {
    const int rc = check_shape(shape);
    if (rc) return rc;
    if (!theta || !w || !c) return MAVG_E_NULL;
    if (k < 1 || layer < 1 || layer > shape->n_layers) return MAVG_E_DIM;
    const Layout y = make_layout(shape, 1);
    if (k > 1 && theta_stride < y.P) return MAVG_E_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (copy_bcast_launch(w, (int64_t)y.d[layer] * y.d[layer - 1], theta + y.w_off[layer], theta_stride, k, s) != 0) return MAVG_E_LAUNCH;
    if (copy_bcast_launch(c, y.d[layer], theta + y.b_off[layer], theta_stride, k, s) != 0) return MAVG_E_LAUNCH;
    return MAVG_OK;
}

extern "C" int32_t dnn_count_correct(const mavg_shape* shape, int32_t k, const float* acts, int64_t act_stride,
                                     const int32_t* labels, int64_t label_stride, int32_t n, int32_t* correct, void* stream) {
    const int rc = check_shape(shape);
    if (rc) return rc;
    if (!acts || !labels || !correct) return MAVG_E_NULL;
    if (k < 1 || n < 1) return MAVG_E_DIM;
    const Layout y = make_layout(shape, n);
    if (k > 1 && (act_stride < y.acts || (label_stride != 0 && label_stride < n))) return MAVG_E_ALIGN;
    if (count_correct_launch(acts + y.a_off[y.L], y.d[y.L], act_stride, labels, label_stride, n, y.d[y.L], k, correct,
                             static_cast<hipStream_t>(stream)) != 0) return MAVG_E_LAUNCH;
    return MAVG_OK;
}
