// Bandwidth/latency-bound kernels around the GEMMs: row softmax, cross-entropy output error,
// column sums with a fused axpby update, and fixed-order reductions.  No atomics anywhere: every sum
// has one owner and a fixed order, so results are reproducible bit for bit.
#include "kernels.h"
#include "gemm.h"
#include "device_math.h"

namespace mavg {

constexpr int kThreads = 256;

__device__ __forceinline__ float block_sum(float v, float* sh) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    const float r = (sh[0] + sh[1]) + (sh[2] + sh[3]);
    __syncthreads();
    return r;
}
__device__ __forceinline__ float block_max(float v, float* sh) {
    v = wave_max(v);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    const float r = fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
    __syncthreads();
    return r;
}

// ---- softmax -------------------------------------------------------------------------------------
// One workgroup per row.  A row of up to 256*ITEMS values is held in registers between the three
// passes (max, sum of exponentials, normalise); longer rows are re-read from memory.
template <int ITEMS>
__global__ __launch_bounds__(kThreads) void softmax_rows_kernel(float* z, int64_t ld, int64_t bstride, int cols) {
    __shared__ float sh[4];
    float* __restrict__ row = z + (int64_t)blockIdx.y * bstride + (int64_t)blockIdx.x * ld;
    const int t = threadIdx.x;
    float v[ITEMS];
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int j = t + i * kThreads;
        v[i] = j < cols ? row[j] : -INFINITY;
        m = fmaxf(m, v[i]);
    }
    m = block_max(m, sh);
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        v[i] = expf(v[i] - m);          // exp(-inf) = 0 for the padding
        s += v[i];
    }
    s = block_sum(s, sh);
    const float inv = 1.f / s;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int j = t + i * kThreads;
        if (j < cols) row[j] = v[i] * inv;
    }
}

__global__ __launch_bounds__(kThreads) void softmax_rows_long_kernel(float* z, int64_t ld, int64_t bstride, int cols) {
    __shared__ float sh[4];
    float* __restrict__ row = z + (int64_t)blockIdx.y * bstride + (int64_t)blockIdx.x * ld;
    float m = -INFINITY;
    for (int j = threadIdx.x; j < cols; j += kThreads) m = fmaxf(m, row[j]);
    m = block_max(m, sh);
    float s = 0.f;
    for (int j = threadIdx.x; j < cols; j += kThreads) s += expf(row[j] - m);
    s = block_sum(s, sh);
    const float inv = 1.f / s;
    for (int j = threadIdx.x; j < cols; j += kThreads) row[j] = expf(row[j] - m) * inv;
}

int softmax_rows_launch(float* z, int64_t ld, int64_t bstride, int rows, int cols, int batch, hipStream_t s) {
    if (rows <= 0 || cols <= 0 || batch <= 0) return 0;
    dim3 grid((unsigned)rows, (unsigned)batch);
    if (cols <= kThreads * 4) hipLaunchKernelGGL(softmax_rows_kernel<4>, grid, dim3(kThreads), 0, s, z, ld, bstride, cols);
    else if (cols <= kThreads * 16) hipLaunchKernelGGL(softmax_rows_kernel<16>, grid, dim3(kThreads), 0, s, z, ld, bstride, cols);
    else if (cols <= kThreads * 36) hipLaunchKernelGGL(softmax_rows_kernel<36>, grid, dim3(kThreads), 0, s, z, ld, bstride, cols);
    else hipLaunchKernelGGL(softmax_rows_long_kernel, grid, dim3(kThreads), 0, s, z, ld, bstride, cols);
    return note_hip_error(hipGetLastError());
}

// ---- cross-entropy output error ------------------------------------------------------------------
// One more row of workgroups than the matrix has rows: workgroup (0, rows, b) gathers p(n, labels[n]) of all rows of
// replica b by itself and sums -log of them in a fixed order (thread-strided partial sums, then the workgroup's tree),
// so the loss needs neither a per-row buffer nor a launch of its own.  p is only read by this launch.
__global__ __launch_bounds__(kThreads) void ce_delta_kernel(const float* __restrict__ p, int64_t ldp, int64_t p_bstride,
                                                            const int32_t* __restrict__ labels, int64_t label_bstride,
                                                            float* __restrict__ delta, int64_t ldd, int64_t d_bstride,
                                                            float* __restrict__ loss_sum, int rows, int cols, float scale) {
    __shared__ float sh[4];
    const int b = blockIdx.z, n = blockIdx.y;
    if (n == rows) {      // (uniform over the workgroup)
        if (blockIdx.x != 0 || loss_sum == nullptr) return;
        float s = 0.f;
        for (int i = threadIdx.x; i < rows; i += kThreads) {
            const int y = labels[(int64_t)b * label_bstride + i];
            if (y >= 0 && y < cols) s += -logf(p[(int64_t)b * p_bstride + (int64_t)i * ldp + y]);
        }
        s = block_sum(s, sh);
        if (threadIdx.x == 0) loss_sum[b] = s;
        return;
    }
    const int y = labels[(int64_t)b * label_bstride + n];
    const float* __restrict__ pr = p + (int64_t)b * p_bstride + (int64_t)n * ldp;
    float* __restrict__ dr = delta + (int64_t)b * d_bstride + (int64_t)n * ldd;
    for (int j = blockIdx.x * kThreads + threadIdx.x; j < cols; j += gridDim.x * kThreads) {
        const float q = pr[j];
        dr[j] = (j == y ? q - 1.f : q) * scale;
    }
}

int ce_delta_launch(const float* p, int64_t ldp, int64_t p_bstride, const int32_t* labels, int64_t label_bstride,
                    float* delta, int64_t ldd, int64_t d_bstride, float* loss_sum, int rows, int cols, int batch,
                    float scale, hipStream_t s) {
    if (rows <= 0 || cols <= 0 || batch <= 0) return 0;
    int gx = (cols + kThreads * 4 - 1) / (kThreads * 4);
    if (gx < 1) gx = 1;
    dim3 grid((unsigned)gx, (unsigned)rows + 1u, (unsigned)batch);
    hipLaunchKernelGGL(ce_delta_kernel, grid, dim3(kThreads), 0, s, p, ldp, p_bstride, labels, label_bstride, delta, ldd,
                       d_bstride, loss_sum, rows, cols, scale);
    return note_hip_error(hipGetLastError());
}

// ---- column sums with fused update ---------------------------------------------------------------
// dst[j] = beta dst[j] + alpha sum_r (X(r, j) - Y(r, j));  dst2[j] += dst[j];  optionally Xcopy(r, j) = X(r, j) and
// sq_partial[workgroup] = sum over the workgroup's 32 columns of (X - Y)^2 (fixed order; the caller adds them up).
// A workgroup owns 32 columns: 1024 threads = 32 columns x 32 row groups; row group g sums rows g, g+32, ...
// top to bottom, eight rows per trip with their loads issued together (a wavefront reads two 128-byte row
// segments per load), then the 32 partial sums of a column are combined in a fixed order through LDS.
constexpr int kColsumGroups = 32;
__global__ __launch_bounds__(32 * kColsumGroups) void colsum_axpby_kernel(const float* __restrict__ X, int64_t ldx,
                                                                         const float* __restrict__ Y, int64_t ldy,
                                                                         float* __restrict__ dst, float* __restrict__ dst2,
                                                                         float* __restrict__ xcopy, int64_t ldc,
                                                                         float* __restrict__ sq_partial,
                                                                         int rows, int cols, float alpha, float beta) {
    __shared__ float sh[kColsumGroups][33];
    __shared__ float sq[kColsumGroups][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int j = blockIdx.x * 32 + tx;
    float s = 0.f, s2 = 0.f;
    if (j < cols) {
        const float* __restrict__ x = X + j;
        const float* __restrict__ y = Y ? Y + j : nullptr;
        int n = ty;
        for (; n + 7 * kColsumGroups < rows; n += 8 * kColsumGroups) {
            float v[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) v[q] = x[(int64_t)(n + kColsumGroups * q) * ldx];
            if (xcopy) {
#pragma unroll
                for (int q = 0; q < 8; ++q) xcopy[(int64_t)(n + kColsumGroups * q) * ldc + j] = v[q];
            }
            if (y) {
#pragma unroll
                for (int q = 0; q < 8; ++q) v[q] -= y[(int64_t)(n + kColsumGroups * q) * ldy];
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) { s += v[q]; s2 += v[q] * v[q]; }
        }
        for (; n < rows; n += kColsumGroups) {
            float v = x[(int64_t)n * ldx];
            if (xcopy) xcopy[(int64_t)n * ldc + j] = v;
            if (y) v -= y[(int64_t)n * ldy];
            s += v;
            s2 += v * v;
        }
    }
    sh[ty][tx] = s;
    sq[ty][tx] = s2;
    __syncthreads();
    if (sq_partial && ty == 1) {          // one wavefront-half: column totals, then across the 32 columns, fixed order
        float c2 = 0.f;
#pragma unroll
        for (int g = 0; g < kColsumGroups; ++g) c2 += sq[g][tx];
        sq[0][tx] = c2;                   // row 0 is read by these same 32 threads only
        __builtin_amdgcn_wave_barrier();
        if (tx == 0) {
            float t2 = 0.f;
            for (int c = 0; c < 32; ++c) t2 += sq[0][c];
            sq_partial[blockIdx.x] = t2;
        }
    }
    if (ty == 0 && j < cols) {
        float tot = 0.f;
#pragma unroll
        for (int g = 0; g < kColsumGroups; ++g) tot += sh[g][tx];
        float r = alpha * tot;
        if (beta != 0.f) r += beta * dst[j];
        dst[j] = r;
        if (dst2) dst2[j] += r;
    }
}

int colsum_blocks(int cols) { return (cols + 31) / 32; }

int colsum_axpby_launch(const float* X, int64_t ldx, const float* Y, int64_t ldy, float* dst, float* dst2, float* xcopy,
                        int64_t ldc, float* sq_partial, int rows, int cols, float alpha, float beta, hipStream_t s) {
    if (cols <= 0) return 0;
    hipLaunchKernelGGL(colsum_axpby_kernel, dim3((unsigned)colsum_blocks(cols)), dim3(32 * kColsumGroups), 0, s, X, ldx, Y, ldy, dst,
                       dst2, xcopy, ldc, sq_partial, rows, cols, alpha, beta);
    return note_hip_error(hipGetLastError());
}

// ---- broadcast copy: dst[b*dst_bstride + i] = src[i] -------------------------------------------------
__global__ __launch_bounds__(kThreads) void copy_bcast_kernel(const float* __restrict__ src, int64_t count,
                                                              float* __restrict__ dst, int64_t dst_bstride) {
    float* d = dst + (int64_t)blockIdx.y * dst_bstride;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < count; i += (int64_t)gridDim.x * kThreads) d[i] = src[i];
}

int copy_bcast_launch(const float* src, int64_t count, float* dst, int64_t dst_bstride, int batch, hipStream_t s) {
    if (count <= 0 || batch <= 0) return 0;
    int64_t gx = (count + kThreads - 1) / kThreads;
    if (gx > 8192) gx = 8192;
    hipLaunchKernelGGL(copy_bcast_kernel, dim3((unsigned)gx, (unsigned)batch), dim3(kThreads), 0, s, src, count, dst, dst_bstride);
    return note_hip_error(hipGetLastError());
}

// ---- frames whose largest posterior is the label's ---------------------------------------------------
__global__ void zero_i32_kernel(int32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// One workgroup per row: arg max over the row (lowest index among equal maxima), compared with the label;
// integer atomic count per batch entry (order-independent, so the result is reproducible).
__global__ __launch_bounds__(kThreads) void argmax_correct_kernel(const float* __restrict__ p, int64_t ld, int64_t bstride,
                                                                  const int32_t* __restrict__ labels, int64_t label_bstride,
                                                                  int cols, int32_t* __restrict__ correct) {
    __shared__ float shv[kThreads / 64];
    __shared__ int shi[kThreads / 64];
    const int row = blockIdx.x, b = blockIdx.y;
    const float* r = p + (int64_t)b * bstride + (int64_t)row * ld;
    float best = -INFINITY;
    int idx = 0x7fffffff;
    for (int j = threadIdx.x; j < cols; j += kThreads) {
        const float v = r[j];
        if (v > best) { best = v; idx = j; }       // ascending j per thread: the first maximum is kept
    }
    for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_down(best, off, 64);
        const int oi = __shfl_down(idx, off, 64);
        if (ov > best || (ov == best && oi < idx)) { best = ov; idx = oi; }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { shv[wave] = best; shi[wave] = idx; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kThreads / 64; ++w)
            if (shv[w] > best || (shv[w] == best && shi[w] < idx)) { best = shv[w]; idx = shi[w]; }
        if (idx == labels[(int64_t)b * label_bstride + row]) atomicAdd(&correct[b], 1);
    }
}

int count_correct_launch(const float* p, int64_t ld, int64_t bstride, const int32_t* labels, int64_t label_bstride,
                         int rows, int cols, int batch, int32_t* correct, hipStream_t s) {
    hipLaunchKernelGGL(zero_i32_kernel, dim3((unsigned)((batch + 63) / 64)), dim3(64), 0, s, correct, batch);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return note_hip_error(e);
    hipLaunchKernelGGL(argmax_correct_kernel, dim3((unsigned)rows, (unsigned)batch), dim3(kThreads), 0, s, p, ld, bstride,
                       labels, label_bstride, cols, correct);
    return note_hip_error(hipGetLastError());
}

}  // namespace mavg
