// placeholder until the bf16 MFMA kernels land
#include "ols_internal.h"
namespace ols {
hipError_t launch_gemm_bf16_fwd(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gemm_bf16_dw(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gemm_bf16_da(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_cast_bf16(const float*, int64_t, uint16_t*, uint16_t*, int, int, int, hipStream_t) { return hipErrorNotSupported; }
}
