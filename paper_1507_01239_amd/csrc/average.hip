// replicas_average: theta_r <- (1/k) sum_j theta_j for k parameter vectors resident in HBM (Sec. 3, eqs. 1-2).
// Pure streaming.  Each thread owns 16-byte columns: it issues its loads back to back, adds them as a balanced
// pairwise tree (a fixed order), scales once and stores.
//   k <= 5 : one pass, k reads + k writes per column.
//   k >= 6 : two passes -- (a) k reads, the mean written to replica 0; (b) replica 0 copied to the other
//            k-1 replicas.  That moves (2k+1)/(2k) of the one-pass bytes, but a read-mostly pass and a
//            write-mostly pass each run close to copy speed, while 2k interleaved read and write streams do
//            not (measured at k = 8, 38.3 M parameters: 0.41 ms against 0.44 ms).
// Workgroups are 64 threads (one wavefront) with two columns per thread, one chunk per workgroup and no
// grid-stride loop: this was the fastest launch shape of those tried.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mavg.h"
#include "gemm.h"

namespace mavg {

constexpr int kAvgBS = 64;     // threads per workgroup
constexpr int kAvgU = 2;       // 16-byte columns per thread

typedef float float4v __attribute__((ext_vector_type(4)));

// Pairwise (balanced tree) sum of v[0..K) into v[0]: ((v0+v1)+(v2+v3))+((v4+v5)+(v6+v7)) for K = 8.
// For K a power of two, identical inputs x give exactly K*x, so identical replicas are returned
// bit for bit after the final multiply by 1/K.
template <int K>
__device__ __forceinline__ void tree_sum(float4v (&v)[K]) {
#pragma unroll
    for (int w = 1; w < K; w *= 2)
#pragma unroll
        for (int j = 0; j + w < K; j += 2 * w) v[j] += v[j + w];
}

// Mean of K replicas for the columns of this workgroup; written to the first NOUT replicas
// (NOUT = K: one-pass averaging; NOUT = 1: first pass of the two-pass form).
template <int K, int NOUT>
__global__ __launch_bounds__(kAvgBS) void average_kernel(float* __restrict__ theta, int64_t stride, int64_t n4, float inv) {
    const int64_t q0 = (int64_t)blockIdx.x * (kAvgBS * kAvgU) + threadIdx.x;
    float4v v[kAvgU][K];
#pragma unroll
    for (int j = 0; j < K; ++j)
#pragma unroll
        for (int u = 0; u < kAvgU; ++u) {
            const int64_t q = q0 + u * kAvgBS;
            v[u][j] = q < n4 ? __builtin_nontemporal_load(reinterpret_cast<const float4v*>(theta + j * stride) + q)
                             : float4v{0.f, 0.f, 0.f, 0.f};
        }
    float4v s[kAvgU];
#pragma unroll
    for (int u = 0; u < kAvgU; ++u) {
        tree_sum<K>(v[u]);
        s[u] = v[u][0] * inv;
    }
#pragma unroll
    for (int j = 0; j < NOUT; ++j)
#pragma unroll
        for (int u = 0; u < kAvgU; ++u) {
            const int64_t q = q0 + u * kAvgBS;
            if (q < n4) {
                float4v* dst = reinterpret_cast<float4v*>(theta + j * stride) + q;
                if (NOUT == 1) *dst = s[u];                       // re-read by the broadcast pass: keep it cacheable
                else __builtin_nontemporal_store(s[u], dst);
            }
        }
}

// 8 < k <= 64, first pass: blocks of 8 replicas are tree-summed, then the (up to 8) block sums are combined as a
// balanced tree too: ((b0+b1)+(b2+b3))+((b4+b5)+(b6+b7)), built with a binary counter of partial sums so
// that only one block of loads is in flight at a time.  The mean goes to replica 0.
__global__ __launch_bounds__(kAvgBS) void average_any_kernel(float* __restrict__ theta, int64_t stride, int64_t n4, int k, float inv) {
    const float4v zero = {0.f, 0.f, 0.f, 0.f};
    const int64_t q = (int64_t)blockIdx.x * kAvgBS + threadIdx.x;
    if (q >= n4) return;
    float4v l0 = zero, l1 = zero, l2 = zero, total = zero;
#pragma unroll 1
    for (int g = 0; g < 8; ++g) {
        float4v v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int r = g * 8 + j;
            v[j] = r < k ? (reinterpret_cast<const float4v*>(theta + r * stride))[q] : zero;
        }
        tree_sum<8>(v);
        float4v b = v[0];
        if ((g & 1) == 0) { l0 = b; continue; }
        b = l0 + b;
        if ((g & 2) == 0) { l1 = b; continue; }
        b = l1 + b;
        if ((g & 4) == 0) { l2 = b; continue; }
        total = l2 + b;
    }
    reinterpret_cast<float4v*>(theta)[q] = total * inv;
}

// second pass: replica 0 -> replicas 1..k-1
__global__ __launch_bounds__(kAvgBS) void average_broadcast_kernel(float* __restrict__ theta, int64_t stride, int64_t n4, int k) {
    const int64_t q0 = (int64_t)blockIdx.x * (kAvgBS * kAvgU) + threadIdx.x;
    float4v s[kAvgU];
#pragma unroll
    for (int u = 0; u < kAvgU; ++u) {
        const int64_t q = q0 + u * kAvgBS;
        s[u] = q < n4 ? reinterpret_cast<const float4v*>(theta)[q] : float4v{0.f, 0.f, 0.f, 0.f};
    }
    for (int j = 1; j < k; ++j)
#pragma unroll
        for (int u = 0; u < kAvgU; ++u) {
            const int64_t q = q0 + u * kAvgBS;
            if (q < n4) __builtin_nontemporal_store(s[u], reinterpret_cast<float4v*>(theta + j * stride) + q);
        }
}

// the last count % 4 elements (same summation tree)
__global__ void average_tail_kernel(float* __restrict__ theta, int64_t stride, int64_t begin, int64_t count, int k, float inv) {
    const int64_t i = begin + threadIdx.x;
    if (i < count) {
        float blk[8];
        for (int g = 0; g < 8; ++g) {
            float v[8];
            for (int j = 0; j < 8; ++j) v[j] = (g * 8 + j < k) ? theta[(int64_t)(g * 8 + j) * stride + i] : 0.f;
            blk[g] = ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
        }
        float s = ((blk[0] + blk[1]) + (blk[2] + blk[3])) + ((blk[4] + blk[5]) + (blk[6] + blk[7]));
        s *= inv;
        for (int j = 0; j < k; ++j) theta[j * stride + i] = s;
    }
}

}  // namespace mavg

using namespace mavg;

extern "C" int32_t replicas_average(float* theta, int64_t theta_stride, int64_t count, int32_t k, void* stream) {
    if (!theta) return MAVG_E_NULL;
    if (count < 0 || k < 1 || k > 64) return MAVG_E_DIM;
    if ((reinterpret_cast<uintptr_t>(theta) & 15u) != 0) return MAVG_E_ALIGN;
    if (k > 1 && (theta_stride < count || (theta_stride & 3) != 0)) return MAVG_E_ALIGN;
    if (count == 0) return MAVG_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const float inv = 1.0f / (float)k;
    const int64_t n4 = count >> 2;
    if (n4 > 0) {
        const int64_t per_wg = kAvgBS * kAvgU;
        const dim3 grid((unsigned)((n4 + per_wg - 1) / per_wg)), block(kAvgBS);
        bool broadcast = false;
        switch (k) {
        case 1: hipLaunchKernelGGL((average_kernel<1, 1>), grid, block, 0, s, theta, theta_stride, n4, inv); break;
        case 2: hipLaunchKernelGGL((average_kernel<2, 2>), grid, block, 0, s, theta, theta_stride, n4, inv); break;
        case 3: hipLaunchKernelGGL((average_kernel<3, 3>), grid, block, 0, s, theta, theta_stride, n4, inv); break;
        case 4: hipLaunchKernelGGL((average_kernel<4, 4>), grid, block, 0, s, theta, theta_stride, n4, inv); break;
        case 5: hipLaunchKernelGGL((average_kernel<5, 5>), grid, block, 0, s, theta, theta_stride, n4, inv); break;
        case 6: hipLaunchKernelGGL((average_kernel<6, 1>), grid, block, 0, s, theta, theta_stride, n4, inv); broadcast = true; break;
        case 7: hipLaunchKernelGGL((average_kernel<7, 1>), grid, block, 0, s, theta, theta_stride, n4, inv); broadcast = true; break;
        case 8: hipLaunchKernelGGL((average_kernel<8, 1>), grid, block, 0, s, theta, theta_stride, n4, inv); broadcast = true; break;
        default:
            hipLaunchKernelGGL(average_any_kernel, dim3((unsigned)((n4 + kAvgBS - 1) / kAvgBS)), block, 0, s, theta, theta_stride, n4,
                               (int)k, inv);
            broadcast = true;
            break;
        }
        if (note_hip_error(hipGetLastError()) != 0) return MAVG_E_LAUNCH;
        if (broadcast) {
            hipLaunchKernelGGL(average_broadcast_kernel, grid, block, 0, s, theta, theta_stride, n4, (int)k);
            if (note_hip_error(hipGetLastError()) != 0) return MAVG_E_LAUNCH;
        }
    }
    if ((count & 3) != 0) {
        hipLaunchKernelGGL(average_tail_kernel, dim3(1), dim3(4), 0, s, theta, theta_stride, n4 << 2, count, (int)k, inv);
        if (note_hip_error(hipGetLastError()) != 0) return MAVG_E_LAUNCH;
    }
    return MAVG_OK;
}
