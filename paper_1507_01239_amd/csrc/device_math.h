// Device-side scalar helpers shared by the kernels of this library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mavg {

__device__ __forceinline__ float sigmoidf_dev(float z) { return 1.f / (1.f + expf(-z)); }

// Philox4x32-10 (Salmon et al., SC'11): ten multiply-xor rounds on a 4x32-bit counter with a 2x32-bit
// key advanced by Weyl constants between rounds.
__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint32_t k0, uint32_t k1) {
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(M0, c.x), lo0 = M0 * c.x;
        const uint32_t hi1 = __umulhi(M1, c.z), lo1 = M1 * c.z;
        c = make_uint4(hi1 ^ c.y ^ k0, lo1, hi0 ^ c.w ^ k1, lo0);
        k0 += W0;
        k1 += W1;
    }
    return c;
}

// Uniform in [0,1) of flat element e: word (e & 3) of the block with counter (e >> 2, step, layer, phase),
// top 24 bits scaled by 2^-24 (exact in float32).
__device__ __forceinline__ float philox_uniform(uint64_t e, uint32_t k0, uint32_t k1, uint32_t step,
                                                uint32_t layer, uint32_t phase) {
    const uint4 r = philox4x32_10(make_uint4((uint32_t)(e >> 2), step, layer, phase), k0, k1);
    const uint32_t sel = (uint32_t)e & 3u;
    const uint32_t w = sel == 0 ? r.x : sel == 1 ? r.y : sel == 2 ? r.z : r.w;
    return (float)(w >> 8) * (1.0f / 16777216.0f);
}

// Wavefront (64 lanes) reductions; every lane receives the result.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

}  // namespace mavg
