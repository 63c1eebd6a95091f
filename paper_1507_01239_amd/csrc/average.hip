// replicas_average: theta_r <- (1/k) sum_j theta_j for k parameter vectors resident in HBM.
// Pure streaming (k reads + k writes per element): each thread owns 16-byte columns, issues the k
// independent loads back to back, adds them in replica order, scales once and stores k copies.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mavg.h"

namespace mavg {

constexpr int kAvgThreads = 256;

typedef float float4v __attribute__((ext_vector_type(4)));

template <int K>
__global__ __launch_bounds__(kAvgThreads) void average_kernel(float* __restrict__ theta, int64_t stride, int64_t n4, float inv) {
    const int64_t step = (int64_t)gridDim.x * kAvgThreads;
    for (int64_t q = (int64_t)blockIdx.x * kAvgThreads + threadIdx.x; q < n4; q += step) {
        float4v v[K];
#pragma unroll
        for (int j = 0; j < K; ++j)
            v[j] = __builtin_nontemporal_load(reinterpret_cast<const float4v*>(theta + j * stride) + q);
        float4v s = v[0];
#pragma unroll
        for (int j = 1; j < K; ++j) s += v[j];
        s *= inv;
#pragma unroll
        for (int j = 0; j < K; ++j)
            __builtin_nontemporal_store(s, reinterpret_cast<float4v*>(theta + j * stride) + q);
    }
}

// any k: two passes over the replicas per column
__global__ __launch_bounds__(kAvgThreads) void average_any_kernel(float* __restrict__ theta, int64_t stride, int64_t n4, int k, float inv) {
    const int64_t step = (int64_t)gridDim.x * kAvgThreads;
    for (int64_t q = (int64_t)blockIdx.x * kAvgThreads + threadIdx.x; q < n4; q += step) {
        float4v s = reinterpret_cast<const float4v*>(theta)[q];
        for (int j = 1; j < k; ++j) s += (reinterpret_cast<const float4v*>(theta + j * stride))[q];
        s *= inv;
        for (int j = 0; j < k; ++j) (reinterpret_cast<float4v*>(theta + j * stride))[q] = s;
    }
}

// the last count % 4 elements
__global__ void average_tail_kernel(float* __restrict__ theta, int64_t stride, int64_t begin, int64_t count, int k, float inv) {
    const int64_t i = begin + threadIdx.x;
    if (i < count) {
        float s = theta[i];
        for (int j = 1; j < k; ++j) s += theta[j * stride + i];
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
        int64_t blocks = (n4 + kAvgThreads - 1) / kAvgThreads;
        const int64_t cap = 256 * 8;    // 8 workgroups per compute unit, grid-stride beyond that
        if (blocks > cap) blocks = cap;
        dim3 grid((unsigned)blocks), block(kAvgThreads);
        switch (k) {
        case 1: hipLaunchKernelGGL(average_kernel<1>, grid, block, 0, s, theta, theta_stride, n4, inv); break;
        case 2: hipLaunchKernelGGL(average_kernel<2>, grid, block, 0, s, theta, theta_stride, n4, inv); break;
        case 3: hipLaunchKernelGGL(average_kernel<3>, grid, block, 0, s, theta, theta_stride, n4, inv); break;
        case 4: hipLaunchKernelGGL(average_kernel<4>, grid, block, 0, s, theta, theta_stride, n4, inv); break;
        case 5: hipLaunchKernelGGL(average_kernel<5>, grid, block, 0, s, theta, theta_stride, n4, inv); break;
        case 6: hipLaunchKernelGGL(average_kernel<6>, grid, block, 0, s, theta, theta_stride, n4, inv); break;
        case 7: hipLaunchKernelGGL(average_kernel<7>, grid, block, 0, s, theta, theta_stride, n4, inv); break;
        case 8: hipLaunchKernelGGL(average_kernel<8>, grid, block, 0, s, theta, theta_stride, n4, inv); break;
        default: hipLaunchKernelGGL(average_any_kernel, grid, block, 0, s, theta, theta_stride, n4, (int)k, inv); break;
        }
        if (hipGetLastError() != hipSuccess) return MAVG_E_LAUNCH;
    }
    if ((count & 3) != 0) {
        hipLaunchKernelGGL(average_tail_kernel, dim3(1), dim3(4), 0, s, theta, theta_stride, n4 << 2, count, (int)k, inv);
        if (hipGetLastError() != hipSuccess) return MAVG_E_LAUNCH;
    }
    return MAVG_OK;
}
