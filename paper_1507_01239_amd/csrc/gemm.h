// Internal C++ interface of the fp32 MFMA GEMM used by every dense contraction of the library.
// Not part of the C ABI (see include/mavg.h for that).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mavg {

// Remember / report the last HIP error a launch of this library saw (per host thread).
int note_hip_error(hipError_t e);   // returns (int)e

// The library is written for MI355X only: 256 compute units in 8 XCDs.
constexpr int kNumCU = 256;
constexpr int kNumXCD = 8;

enum EpiKind : int {
    EPI_STORE = 0,            // C = v
    EPI_BIAS = 1,             // C = v + bias[n]
    EPI_BIAS_SIGMOID = 2,     // C = alpha * sigmoid(v + bias[n])
    EPI_MUL_DSIGMOID = 3,     // C = v * a * (1 - a),  a = aux[m, n]
    EPI_AXPBY = 4,            // C = beta*C + alpha*v ;  if C2: C2 += C
    EPI_BIAS_SIGMOID_SAMPLE = 5,  // p = sigmoid(v + bias[n]); if C: C = p;  C2 = [u(m*N+n) < p]
    EPI_ROWSCALE_ADD = 6,     // C = alpha*v + rowvec[m] * aux[m, n]
};

struct Epilogue {
    int kind = EPI_STORE;
    const float* bias = nullptr; int64_t bias_bstride = 0;
    const float* aux = nullptr;  int64_t ldaux = 0; int64_t aux_bstride = 0;
    float* C2 = nullptr;         int64_t ldc2 = 0;  int64_t c2_bstride = 0;
    float alpha = 1.f, beta = 0.f;
    // EPI_BIAS_SIGMOID / EPI_MUL_DSIGMOID with tanh in place of the sigmoid: C = tanh(v + bias[n]) / C = v * (1 - a^2)
    int act_tanh = 0;
    // optional device-side factors of alpha (EPI_AXPBY): alpha_eff = alpha * alpha_dev0[b] * alpha_dev1[b]
    const float* alpha_dev0 = nullptr; const float* alpha_dev1 = nullptr;
    const float* rowvec = nullptr; int64_t rowvec_bstride = 0;     // EPI_ROWSCALE_ADD
    // optional (EPI_AXPBY): output column `lastcol` is not part of C but a separate vector, lastcol_dst[b][m]
    // (a weight matrix whose bias is the gradient's extra column)
    int lastcol = -1; float* lastcol_dst = nullptr; int64_t lastcol_bstride = 0;
    // optional, only for an m-contiguous A operand (forces an unsplit contraction):
    //   rowsum_dst[b][m] = rowsum_beta * rowsum_dst[b][m] + rowsum_alpha * sum_k A(m,k)
    //   if rowsum_dst2: rowsum_dst2[b][m] += rowsum_dst[b][m]   (a bias next to its momentum vector)
    float* rowsum_dst = nullptr; int64_t rowsum_bstride = 0; float rowsum_alpha = 1.f, rowsum_beta = 0.f;
    float* rowsum_dst2 = nullptr; int64_t rowsum2_bstride = 0;
    //   rowsum_w (optional): weights of the sum, sum_k A(m,k) * rowsum_w[b][k] (a matrix-vector product next to the
    //   matrix-matrix one: the bias gradient when the "ones" column has been preconditioned); the factors
    //   alpha_dev0[b] * alpha_dev1[b] of alpha apply to rowsum_alpha as well
    const float* rowsum_w = nullptr; int64_t rowsum_w_bstride = 0;
    // optional, a short vector summed on the side of the launch (forces an unsplit contraction, not taken by the
    // in-workgroup-split kernels): side_sum_dst[0] = sum_{i < side_sum_n} side_sum_src[i], by workgroup 0 of batch
    // element 0 behind its own tile, in the order of a 256-thread fixed-order segment sum (thread-strided partial
    // sums, then the four wavefronts' sums pairwise) - e.g. the per-block squared errors a preceding launch left
    const float* side_sum_src = nullptr; float* side_sum_dst = nullptr; int side_sum_n = 0;
    uint32_t key0 = 0, key1 = 0, step = 0, layer = 0, phase = 0;   // Philox stream of the sampling epilogue
};

// C[b](m,n) = epilogue( sum_k A[b](m,k) * B[b](k,n) ),  b in [0,batch).
//   a_kc: A(m,k) = A[m*lda + k]  (contraction index contiguous) else A[k*lda + m]
//   b_kc: B(k,n) = B[n*ldb + k]  else B[k*ldb + n]
//   C(m,n) = C[m*ldc + n]
struct GemmDesc {
    const float* A = nullptr; int64_t lda = 0; int64_t a_bstride = 0; bool a_kc = true;
    const float* B = nullptr; int64_t ldb = 0; int64_t b_bstride = 0; bool b_kc = true;
    float* C = nullptr;       int64_t ldc = 0; int64_t c_bstride = 0;
    int M = 0, N = 0, K = 0, batch = 1;
    // For an operand whose m (or n) index is the contiguous one: its rows may be READ up to the next multiple of 4
    // columns (the caller's buffer has that padding inside its row stride; what it holds is never used in a
    // stored result).  Lets the direct-to-LDS kernel take widths that are not multiples of 4.
    bool a_pad4 = false, b_pad4 = false;
    Epilogue epi;
    int force_cfg = -1;     // -1: choose; otherwise tile configuration index
    int force_splits = 0;   // 0: choose; otherwise number of contraction splits
};

// Kernel / tile configurations (also the `cfg` argument of the exported mavg_gemm).
enum GemmCfg : int {
    CFG_AUTO = -1,
    CFG_64 = 0,          // 64x64 tiles, 2x2 wavefronts of 32x32: direct-to-LDS (ring of four stages) whenever the operands allow
    CFG_64_REG = 1,      // 64x64 tiles, always register-staged (guarded loads: any shape, any alignment)
    CFG_128_REG = 2,     // 128x128 tiles, 2x4 wavefronts of 64x32, register-staged
    CFG_128x64 = 3,      // direct-to-LDS only from here on (replanned as CFG_64_REG when the operands do not allow it):
    CFG_64x128 = 4,      //   2x2 wavefronts of 64x32 / 32x64 / 64x64
    CFG_128 = 5,
    CFG_64_RING3 = 6,    // as CFG_64 with a ring of three LDS stages
    CFG_KG_32x64 = 7,    // 32x64 tile, contraction split four ways inside the workgroup
    CFG_KG_32x32 = 8,    // 32x32 tile, likewise, one wavefront per k-group (no barrier in the loop)
    CFG_COUNT = 9
};

struct GemmPlan { int cfg; int splits; int bm, bn; };

GemmPlan gemm_plan(int M, int N, int K, int batch, int force_cfg, int force_splits);
// float32 elements of scratch the plan for this problem needs (0 when it is not split)
int64_t gemm_ws_floats(int M, int N, int K, int batch, int force_cfg = -1, int force_splits = 0);
// enqueue; returns hipError_t as int (0 = ok).  ws must hold gemm_ws_floats() floats when that is > 0.
int gemm_launch(const GemmDesc& d, float* ws, int64_t ws_floats, hipStream_t stream);

// Several independent GEMMs of the same operand layouts and batch count in ONE launch (64x64 tiles, unsplit
// contraction, no scratch).  `thin`: products with few output columns and a long contraction, both operands
// k-contiguous (32x32 tiles, the contraction split four ways inside each workgroup).  Returns hipError_t as int.
constexpr int kThinMaxProblems = 40;    // thin problems one launch takes (more are launched in further launches)
int gemm_launch_grouped(const GemmDesc* d, int count, hipStream_t stream, bool thin = false);

}  // namespace mavg
