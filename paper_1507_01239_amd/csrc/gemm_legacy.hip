// Register-staged GEMM kernels (guarded loads: any alignment, any raggedness), single and grouped.
#include "gemm_launchers.h"

namespace mavg {

template <int BM, int BN, int BK, int WM, int WN, int PF>
static void launch_cfg(const GemmKParams& p, bool a_kc, bool b_kc, dim3 grid, hipStream_t s) {
    const dim3 block(64 * WM * WN);
    if (a_kc && b_kc) hipLaunchKernelGGL((gemm_kernel<BM, BN, BK, WM, WN, PF, true, true>), grid, block, 0, s, p);
    else if (a_kc && !b_kc) hipLaunchKernelGGL((gemm_kernel<BM, BN, BK, WM, WN, PF, true, false>), grid, block, 0, s, p);
    else if (!a_kc && !b_kc) hipLaunchKernelGGL((gemm_kernel<BM, BN, BK, WM, WN, PF, false, false>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((gemm_kernel<BM, BN, BK, WM, WN, PF, false, true>), grid, block, 0, s, p);
}

void launch_legacy(bool big, const GemmKParams& p, bool a_kc, bool b_kc, dim3 grid, hipStream_t s) {
    if (big) launch_cfg<128, 128, 16, 2, 4, 4>(p, a_kc, b_kc, grid, s);
    else launch_cfg<64, 64, 16, 2, 2, 4>(p, a_kc, b_kc, grid, s);
}

void launch_grouped_legacy(const GemmGroupParams& gp, bool a_kc, bool b_kc, dim3 grid, hipStream_t s) {
    const dim3 block(256);
    if (a_kc && b_kc) hipLaunchKernelGGL((gemm_grouped_kernel<64, 64, 16, 2, 2, 4, true, true>), grid, block, 0, s, gp);
    else if (a_kc && !b_kc) hipLaunchKernelGGL((gemm_grouped_kernel<64, 64, 16, 2, 2, 4, true, false>), grid, block, 0, s, gp);
    else if (!a_kc && !b_kc) hipLaunchKernelGGL((gemm_grouped_kernel<64, 64, 16, 2, 2, 4, false, false>), grid, block, 0, s, gp);
    else hipLaunchKernelGGL((gemm_grouped_kernel<64, 64, 16, 2, 2, 4, false, true>), grid, block, 0, s, gp);
}

}  // namespace mavg
