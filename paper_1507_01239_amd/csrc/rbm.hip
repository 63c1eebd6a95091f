// rbm_cd1_step: one CD-1 minibatch update of an RBM.  Three affine GEMMs (hidden probabilities with
// the Bernoulli sampling fused into the epilogue, reconstruction, hidden probabilities of the
// reconstruction), ONE statistics GEMM fused with the momentum updates of W and of the hidden bias
// (positive minus negative phase as one contraction over the stacked rows [P_h0; -P_h1] and [V0; V1]), a
// column-sum kernel for the visible bias that also stacks V0 and sums the squared reconstruction error per block of
// columns, and a fixed-order sum of those.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "../../include/mavg.h"
#include "gemm.h"
#include "kernels.h"
#include "device_math.h"

using namespace mavg;

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

struct RbmWs {
    int64_t ldh, ldv;
    int64_t off_ph, off_h0, off_vv, off_part, off_gemm, gemm_floats, total;     // ph: [P_h0; -P_h1], vv: [V0; V1], 2n rows each
};

RbmWs rbm_ws(int V, int H, int n) {
    RbmWs w;
    w.ldh = round_up(H, 4);
    w.ldv = round_up(V, 4);
    int64_t g = gemm_ws_floats(n, H, V, 1), f;
    f = gemm_ws_floats(n, V, H, 1); if (f > g) g = f;
    w.gemm_floats = round_up(g, 64);
    int64_t off = 0;
    w.off_ph = off;  off += round_up((int64_t)2 * n * w.ldh, 64);
    w.off_h0 = off;  off += round_up((int64_t)n * w.ldh, 64);
    w.off_vv = off;  off += round_up((int64_t)2 * n * w.ldv, 64);
    w.off_part = off; off += round_up(colsum_blocks(V), 64);
    w.off_gemm = off; off += w.gemm_floats;
    w.total = off;
    return w;
}

float* ws_base(void* workspace) {
    return reinterpret_cast<float*>((reinterpret_cast<uintptr_t>(workspace) + 255u) & ~uintptr_t(255));
}

}  // namespace

extern "C" int64_t rbm_workspace_bytes(int32_t n_vis, int32_t n_hid, int32_t n) {
    if (n_vis < 1 || n_hid < 1 || n < 1) return MAVG_E_DIM;
    return rbm_ws(n_vis, n_hid, n).total * 4 + 256;
}

// Where rbm_cd1_step leaves its intermediate matrices: byte offsets from the 256-byte aligned workspace base and row
// strides in floats.
extern "C" int32_t rbm_workspace_layout(int32_t n_vis, int32_t n_hid, int32_t n, int64_t* out) {
    if (!out) return MAVG_E_NULL;
    if (n_vis < 1 || n_hid < 1 || n < 1) return MAVG_E_DIM;
    const RbmWs w = rbm_ws(n_vis, n_hid, n);
    out[0] = w.off_ph * 4;                               out[1] = w.ldh;     // P_h0
    out[2] = w.off_h0 * 4;                               out[3] = w.ldh;     // H0
    out[4] = (w.off_vv + (int64_t)n * w.ldv) * 4;        out[5] = w.ldv;     // V1
    out[6] = (w.off_ph + (int64_t)n * w.ldh) * 4;        out[7] = w.ldh;     // -P_h1
    return MAVG_OK;
}

extern "C" int32_t rbm_hidden_prob(int32_t n_vis, int32_t n_hid, const float* w, const float* c, const float* v,
                                   int32_t n, float* out, void* workspace, int64_t workspace_bytes, void* stream) {
    if (!w || !c || !v || !out) return MAVG_E_NULL;
    if (n_vis < 1 || n_hid < 1 || n < 1) return MAVG_E_DIM;
    if (!aligned16(w) || !aligned16(c) || !aligned16(v) || !aligned16(out)) return MAVG_E_ALIGN;
    const RbmWs lay = rbm_ws(n_vis, n_hid, n);
    if (!workspace || workspace_bytes < lay.total * 4 + 256) return MAVG_E_WORKSPACE;
    float* ws = ws_base(workspace);
    GemmDesc g;
    g.M = n; g.N = n_hid; g.K = n_vis;
    g.A = v; g.lda = n_vis; g.a_kc = true;
    g.B = w; g.ldb = n_vis; g.b_kc = true;
    g.C = out; g.ldc = n_hid;
    g.epi.kind = EPI_BIAS_SIGMOID; g.epi.bias = c;
    if (gemm_launch(g, ws + lay.off_gemm, lay.gemm_floats, static_cast<hipStream_t>(stream)) != 0) return MAVG_E_LAUNCH;
    return MAVG_OK;
}

namespace {

// Host-side checks shared by the two CD-1 entry points (everything except the workspace).
int cd1_check(int32_t V, int32_t H, int32_t vis_type, const float* w, const float* a, const float* c, const float* mw,
              const float* ma, const float* mc, const float* v0, int32_t n, uint32_t flags) {
    if (!w || !a || !c || !mw || !ma || !mc || !v0) return MAVG_E_NULL;
    if (V < 1 || H < 1 || n < 1) return MAVG_E_DIM;
    if (vis_type != MAVG_VIS_BERNOULLI && vis_type != MAVG_VIS_GAUSSIAN) return MAVG_E_FLAG;
    if (flags & ~MAVG_SAMPLE_V1) return MAVG_E_FLAG;
    if ((flags & MAVG_SAMPLE_V1) && vis_type == MAVG_VIS_GAUSSIAN) return MAVG_E_FLAG;
    if (!aligned16(w) || !aligned16(a) || !aligned16(c) || !aligned16(mw) || !aligned16(ma) || !aligned16(mc) ||
        !aligned16(v0))
        return MAVG_E_ALIGN;
    return MAVG_OK;
}

// The launches of one CD-1 step; ws: 256-byte aligned scratch of rbm_ws(V, H, n).total floats, contents undefined on
// entry (every element that a stored result depends on is written before it is read).
int32_t cd1_run(int32_t V, int32_t H, int32_t vis_type, float* w, float* a, float* c, float* mw, float* ma, float* mc,
                const float* v0, int32_t n, float lr, float momentum, uint64_t seed, uint32_t step, uint32_t layer,
                uint32_t flags, float* recon_err, const RbmWs& lay, float* ws, hipStream_t s) {
    float* ph0 = ws + lay.off_ph;                       // rows 0..n-1 of the stacked hidden statistics
    float* ph1 = ph0 + (int64_t)n * lay.ldh;            // rows n..2n-1, stored NEGATED
    float* h0 = ws + lay.off_h0;
    float* vv = ws + lay.off_vv;                        // rows 0..n-1: copy of V0; rows n..2n-1: V1
    float* v1 = vv + (int64_t)n * lay.ldv;
    float* gws = ws + lay.off_gemm;
    const uint32_t k0 = (uint32_t)(seed & 0xFFFFFFFFu), k1 = (uint32_t)(seed >> 32);
    const float invn = 1.0f / (float)n;

    {   // P_h0 = sigmoid(V0 W^T + c), H0 = [u < P_h0]
        GemmDesc g;
        g.M = n; g.N = H; g.K = V;
        g.A = v0; g.lda = V; g.a_kc = true;
        g.B = w; g.ldb = V; g.b_kc = true;
        g.C = ph0; g.ldc = lay.ldh;
        g.epi.kind = EPI_BIAS_SIGMOID_SAMPLE; g.epi.bias = c;
        g.epi.C2 = h0; g.epi.ldc2 = lay.ldh;
        g.epi.key0 = k0; g.epi.key1 = k1; g.epi.step = step; g.epi.layer = layer; g.epi.phase = 0;
        if (gemm_launch(g, gws, lay.gemm_floats, s) != 0) return MAVG_E_LAUNCH;
    }
    {   // V1 from H0 W + a
        GemmDesc g;
        g.M = n; g.N = V; g.K = H;
        g.A = h0; g.lda = lay.ldh; g.a_kc = true;
        g.B = w; g.ldb = V; g.b_kc = false;
        g.C = v1; g.ldc = lay.ldv;
        g.epi.bias = a;
        if (vis_type == MAVG_VIS_GAUSSIAN) g.epi.kind = EPI_BIAS;
        else if (!(flags & MAVG_SAMPLE_V1)) g.epi.kind = EPI_BIAS_SIGMOID;
        else {
            g.epi.kind = EPI_BIAS_SIGMOID_SAMPLE;
            g.C = nullptr;
            g.epi.C2 = v1; g.epi.ldc2 = lay.ldv;
            g.epi.key0 = k0; g.epi.key1 = k1; g.epi.step = step; g.epi.layer = layer; g.epi.phase = 1;
        }
        if (gemm_launch(g, gws, lay.gemm_floats, s) != 0) return MAVG_E_LAUNCH;
    }
    {   // -P_h1 = -sigmoid(V1 W^T + c)
        GemmDesc g;
        g.M = n; g.N = H; g.K = V;
        g.A = v1; g.lda = lay.ldv; g.a_kc = true;
        g.B = w; g.ldb = V; g.b_kc = true;
        g.C = ph1; g.ldc = lay.ldh;
        g.epi.kind = EPI_BIAS_SIGMOID; g.epi.bias = c; g.epi.alpha = -1.f;
        if (gemm_launch(g, gws, lay.gemm_floats, s) != 0) return MAVG_E_LAUNCH;
    }
    // Ma <- momentum Ma + (lr/n) colsum(V0 - V1); a <- a + Ma;  the same pass copies V0 under V1's rows' stride
    // and leaves the squared reconstruction error of each block of 32 columns (summed in block order by the launch below)
    if (colsum_axpby_launch(v0, V, v1, lay.ldv, ma, a, vv, lay.ldv, recon_err ? ws + lay.off_part : nullptr, n, V, lr * invn,
                            momentum, s) != 0) return MAVG_E_LAUNCH;
    {   // MW <- momentum MW + (lr/n) (P_h0^T V0 - P_h1^T V1) = momentum MW + (lr/n) [P_h0; -P_h1]^T [V0; V1];  W <- W + MW
        GemmDesc g;
        g.M = H; g.N = V; g.K = 2 * n;
        g.A = ph0; g.lda = lay.ldh; g.a_kc = false;
        g.a_pad4 = true;        // rows of the stacked statistics are ldh = round_up(H, 4) floats long
        g.B = vv; g.ldb = lay.ldv; g.b_kc = false;
        g.b_pad4 = true;
        g.C = mw; g.ldc = V;
        g.epi.kind = EPI_AXPBY; g.epi.alpha = lr * invn; g.epi.beta = momentum;
        g.epi.C2 = w; g.epi.ldc2 = V;
        // Mc <- momentum Mc + (lr/n) colsum(P_h0 - P_h1), the row sums of this product's first operand;  c <- c + Mc
        g.epi.rowsum_dst = mc; g.epi.rowsum_alpha = lr * invn; g.epi.rowsum_beta = momentum;
        g.epi.rowsum_dst2 = c;
        if (recon_err) {      // the reconstruction error: the blocks' squared errors, summed in block order on the side of this launch
            g.epi.side_sum_src = ws + lay.off_part; g.epi.side_sum_dst = recon_err; g.epi.side_sum_n = colsum_blocks(V);
        }
        if (gemm_launch(g, gws, lay.gemm_floats, s) != 0) return MAVG_E_LAUNCH;
    }
    return MAVG_OK;
}

}  // namespace

extern "C" int32_t rbm_cd1_step(int32_t V, int32_t H, int32_t vis_type, float* w, float* a, float* c, float* mw,
                                float* ma, float* mc, const float* v0, int32_t n, float lr, float momentum,
                                uint64_t seed, uint32_t step, uint32_t layer, uint32_t flags, float* recon_err,
                                void* workspace, int64_t workspace_bytes, void* stream) {
    const int rc = cd1_check(V, H, vis_type, w, a, c, mw, ma, mc, v0, n, flags);
    if (rc) return rc;
    const RbmWs lay = rbm_ws(V, H, n);
    if (!workspace || workspace_bytes < lay.total * 4 + 256) return MAVG_E_WORKSPACE;
    return cd1_run(V, H, vis_type, w, a, c, mw, ma, mc, v0, n, lr, momentum, seed, step, layer, flags, recon_err, lay,
                   ws_base(workspace), static_cast<hipStream_t>(stream));
}

// ---- CD-1 without a workspace argument ----------------------------------------------------------------
// For callers that cannot allocate (code under HIP graph capture, serving loops that own no scratch memory): the
// same step with its scratch in a static device array.  Every device the library runs on holds the array from
// module load to process end; its device address is looked up once per device and kept.
namespace {

constexpr int64_t kStaticScratchBytes = MAVG_RBM_STATIC_SCRATCH_BYTES;       // 32 MiB: covers 2048 x 2048 up to minibatch 512
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices] = {};     // per device: where that device's copy of `scratch` lives

// Device address of the current device's scratch array (nullptr and a noted HIP error on failure).
float* static_scratch() {
    int dev = -1;
    if (note_hip_error(hipGetDevice(&dev)) != 0 || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (note_hip_error(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) != 0) return nullptr;
        g_scratch_ptr[dev] = static_cast<float*>(p);
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" int32_t rbm_cd1_step_static(int32_t V, int32_t H, int32_t vis_type, float* w, float* a, float* c, float* mw,
                                       float* ma, float* mc, const float* v0, int32_t n, float lr, float momentum,
                                       uint64_t seed, uint32_t step, uint32_t layer, uint32_t flags, float* recon_err,
                                       void* stream) {
    const int rc = cd1_check(V, H, vis_type, w, a, c, mw, ma, mc, v0, n, flags);
    if (rc) return rc;
    const RbmWs lay = rbm_ws(V, H, n);
    if (lay.total * 4 > kStaticScratchBytes) return MAVG_E_WORKSPACE;       // before anything touches the device
    float* ws = static_scratch();
    if (!ws) return MAVG_E_LAUNCH;
    return cd1_run(V, H, vis_type, w, a, c, mw, ma, mc, v0, n, lr, momentum, seed, step, layer, flags, recon_err, lay, ws,
                   static_cast<hipStream_t>(stream));
}

// ---- the generator by itself ------------------------------------------------------------------------
namespace mavg {
__global__ __launch_bounds__(256) void philox_fill_kernel(uint32_t* __restrict__ out, int64_t nblocks, uint32_t first,
                                                          uint32_t k0, uint32_t k1, uint32_t step, uint32_t layer, uint32_t phase) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nblocks; i += (int64_t)gridDim.x * 256) {
        const uint4 r = philox4x32_10(make_uint4(first + (uint32_t)i, step, layer, phase), k0, k1);
        reinterpret_cast<uint4*>(out)[i] = r;
    }
}
}  // namespace mavg

extern "C" int32_t mavg_philox_fill(uint32_t* out, int64_t nblocks, uint32_t first_block, uint64_t seed, uint32_t step,
                                    uint32_t layer, uint32_t phase, void* stream) {
    if (!out) return MAVG_E_NULL;
    if (nblocks < 0 || nblocks > ((int64_t)1 << 32)) return MAVG_E_DIM;
    if (!aligned16(out)) return MAVG_E_ALIGN;
    if (nblocks == 0) return MAVG_OK;
    int64_t gx = (nblocks + 255) / 256;
    if (gx > 4096) gx = 4096;
    hipLaunchKernelGGL(philox_fill_kernel, dim3((unsigned)gx), dim3(256), 0, static_cast<hipStream_t>(stream), out, nblocks,
                       first_block, (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32), step, layer, phase);
    return note_hip_error(hipGetLastError()) == 0 ? MAVG_OK : MAVG_E_LAUNCH;
}
