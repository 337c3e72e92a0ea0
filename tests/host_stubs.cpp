// Kernel launchers replaced by no-ops: lets the host side of the library (argument validation,
// launch planning, the workgroup -> tile map) be built without device code and run under
// the address and undefined-behaviour sanitizers on a machine without a GPU.
#include "tess_internal.h"

namespace tess {
hipError_t launch_generic(const GemmArgs&, hipStream_t) { return hipSuccess; }
hipError_t launch_mfma(const GemmArgs&, const Plan&, hipStream_t) { return hipSuccess; }
hipError_t launch_mfma_probe(float*, int, int, int, hipStream_t) { return hipSuccess; }
hipError_t launch_row_sums(const void*, int64_t, int64_t, int64_t, int, int, float*, hipStream_t) { return hipSuccess; }
hipError_t launch_row_sums_bwd(const void*, const void*, int64_t, int64_t, int64_t, int64_t, int, int, float*,
                               hipStream_t) { return hipSuccess; }
hipError_t launch_layernorm_bwd(const void*, const void*, int64_t, int64_t, int64_t, int64_t, int, const float*,
                                const float*, float, float, void*, int64_t, hipStream_t) { return hipSuccess; }
hipError_t launch_normalize(const void*, int64_t, int64_t, int64_t, int, const float*, float, float, void*, int64_t,
                            hipStream_t) { return hipSuccess; }
}  // namespace tess
