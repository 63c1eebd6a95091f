// Direct-to-LDS GEMM kernels with 128x64, 64x128 and 128x128 tiles (problems large in all three dimensions).
#include "gemm_launchers.h"

namespace mavg {

template <int TM, int TN, int NST>
static void launch_dma_t(const GemmKParams& p, bool a_kc, bool b_kc, dim3 grid, hipStream_t s) {
    const dim3 block(256);
    if (a_kc && b_kc) hipLaunchKernelGGL((gemm_dma_kernel<TM, TN, NST, true, true>), grid, block, 0, s, p);
    else if (a_kc && !b_kc) hipLaunchKernelGGL((gemm_dma_kernel<TM, TN, NST, true, false>), grid, block, 0, s, p);
    else if (!a_kc && !b_kc) hipLaunchKernelGGL((gemm_dma_kernel<TM, TN, NST, false, false>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((gemm_dma_kernel<TM, TN, NST, false, true>), grid, block, 0, s, p);
}

void launch_dma128(int cfg, const GemmKParams& p, bool a_kc, bool b_kc, dim3 grid, hipStream_t s) {
    if (cfg == CFG_128x64) launch_dma_t<2, 1, 4>(p, a_kc, b_kc, grid, s);
    else if (cfg == CFG_64x128) launch_dma_t<1, 2, 4>(p, a_kc, b_kc, grid, s);
    else launch_dma_t<2, 2, 4>(p, a_kc, b_kc, grid, s);
}

}  // namespace mavg
