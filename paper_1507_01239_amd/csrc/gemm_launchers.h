// Launch wrappers of the GEMM kernel families.  Each family is instantiated in a translation unit of its own
// (gemm_legacy.hip, gemm_dma64.hip, gemm_dma128.hip, gemm_kg.hip); gemm.hip plans and dispatches.
#pragma once
#include "gemm_device.h"

namespace mavg {

// register-staged kernels: 128x128 tiles with 8 wavefronts (big = true) or 64x64 tiles with 4
void launch_legacy(bool big, const GemmKParams& p, bool a_kc, bool b_kc, dim3 grid, hipStream_t s);
void launch_grouped_legacy(const GemmGroupParams& gp, bool a_kc, bool b_kc, dim3 grid, hipStream_t s);
// direct-to-LDS kernels: 64x64 tiles with a ring of 4 (cfg 1) or 3 (cfg 12) stages; 128x64, 64x128, 128x128 (cfg 9, 10, 11)
void launch_dma64(int cfg, const GemmKParams& p, bool a_kc, bool b_kc, dim3 grid, hipStream_t s);
void launch_dma128(int cfg, const GemmKParams& p, bool a_kc, bool b_kc, dim3 grid, hipStream_t s);
void launch_grouped_dma(const GemmGroupParams& gp, bool a_kc, bool b_kc, dim3 grid, hipStream_t s);
// contraction split inside the workgroup: 32x64 tiles (cfg 13) or 32x32 tiles (cfg 14); thin grouped problems
void launch_kg(int cfg, const GemmKParams& p, bool a_kc, bool b_kc, dim3 grid, hipStream_t s);
void launch_thin(const ThinGroupParams& gp, dim3 grid, hipStream_t s);

}  // namespace mavg
