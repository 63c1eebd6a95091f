// Direct-to-LDS GEMM kernels with 64x64 tiles: the kernels of the training step (single problems with a ring of
// four or three LDS stages, and the grouped launch of the weight gradients with three).
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

void launch_dma64(int cfg, const GemmKParams& p, bool a_kc, bool b_kc, dim3 grid, hipStream_t s) {
    if (cfg == CFG_64_RING3) launch_dma_t<1, 1, 3>(p, a_kc, b_kc, grid, s);
    else launch_dma_t<1, 1, 4>(p, a_kc, b_kc, grid, s);
}

// Ring of the grouped launch: three stages (24 KB of LDS per workgroup, six workgroups per compute unit) measured
// faster than four for the short contractions of the weight gradients.
constexpr int kGroupedStages = 3;

void launch_grouped_dma(const GemmGroupParams& gp, bool a_kc, bool b_kc, dim3 grid, hipStream_t s) {
    const dim3 block(256);
    if (a_kc && b_kc) hipLaunchKernelGGL((gemm_dma_grouped_kernel<1, 1, kGroupedStages, true, true>), grid, block, 0, s, gp);
    else if (a_kc && !b_kc) hipLaunchKernelGGL((gemm_dma_grouped_kernel<1, 1, kGroupedStages, true, false>), grid, block, 0, s, gp);
    else if (!a_kc && !b_kc) hipLaunchKernelGGL((gemm_dma_grouped_kernel<1, 1, kGroupedStages, false, false>), grid, block, 0, s, gp);
    else hipLaunchKernelGGL((gemm_dma_grouped_kernel<1, 1, kGroupedStages, false, true>), grid, block, 0, s, gp);
}

}  // namespace mavg
