// Direct-to-LDS GEMM kernels that split the contraction inside the workgroup (skinny problems), and the grouped
// launch of thin products built on the same body.
#include "gemm_launchers.h"

namespace mavg {

template <int GW>
static void launch_kg_t(const GemmKParams& p, bool a_kc, bool b_kc, dim3 grid, hipStream_t s) {
    const dim3 block(64 * kKGroups * GW);
    if (a_kc && b_kc) hipLaunchKernelGGL((gemm_dma_kg_kernel<GW, true, true>), grid, block, 0, s, p);
    else if (a_kc && !b_kc) hipLaunchKernelGGL((gemm_dma_kg_kernel<GW, true, false>), grid, block, 0, s, p);
    else if (!a_kc && !b_kc) hipLaunchKernelGGL((gemm_dma_kg_kernel<GW, false, false>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((gemm_dma_kg_kernel<GW, false, true>), grid, block, 0, s, p);
}

void launch_kg(int cfg, const GemmKParams& p, bool a_kc, bool b_kc, dim3 grid, hipStream_t s) {
    if (cfg == CFG_KG_32x64) launch_kg_t<2>(p, a_kc, b_kc, grid, s);
    else launch_kg_t<1>(p, a_kc, b_kc, grid, s);
}

void launch_thin(const ThinGroupParams& gp, dim3 grid, hipStream_t s) {
    hipLaunchKernelGGL((gemm_thin_grouped_kernel<kThinKGroups>), grid, dim3(64 * kThinKGroups), 0, s, gp);
}

}  // namespace mavg
