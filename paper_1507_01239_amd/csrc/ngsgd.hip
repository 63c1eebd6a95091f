// NG-SGD preconditioner -- placeholder translation unit while the DNN path is brought up.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mavg.h"
#include "ng_internal.h"

namespace mavg {
int64_t ng_dnn_ws_floats(const int*, int, int, int, int) { return 0; }
int ng_layer_update(const NgLayerArgs&, hipStream_t) { return (int)hipErrorNotSupported; }
}  // namespace mavg

extern "C" int64_t ngsgd_state_bytes(int32_t dim, int32_t rank) {
    if (dim < 2 || rank < 1 || rank > 64 || rank >= dim) return MAVG_E_DIM;
    const int64_t ld = (dim + 3) / 4 * 4;
    return (int64_t)rank * ld * 4 + (int64_t)rank * 8 + 16;
}
extern "C" int64_t ngsgd_workspace_bytes(int32_t, int32_t, int32_t) { return MAVG_E_FLAG; }
extern "C" int32_t ngsgd_state_init(void*, int32_t, int32_t, void*) { return MAVG_E_FLAG; }
extern "C" int32_t ngsgd_precondition(void*, int32_t, int32_t, float*, int64_t, int32_t, float, float, int32_t, void*, int64_t, void*) { return MAVG_E_FLAG; }
