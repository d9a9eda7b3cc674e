#include "qeft_internal.h"
namespace qeft {
bool gemm_fwd_supported(const Layer&, int64_t) { return false; }
hipError_t gemm_fwd(const Layer&, const __half*, int64_t, int64_t, __half*, int64_t, hipStream_t) { return hipErrorNotSupported; }
bool gemm_dx_supported(const Layer&, int64_t) { return false; }
hipError_t gemm_dx(const Layer&, const __half*, int64_t, int64_t, __half*, int64_t, hipStream_t) { return hipErrorNotSupported; }
bool weak_grad_mfma_supported(int, int, int64_t) { return false; }
size_t weak_grad_mfma_workspace(int, int, int64_t) { return 0; }
hipError_t weak_grad_mfma(int, int, const __half*, int64_t, int64_t, const __half*, int64_t, void*, int, int, void*, hipStream_t) { return hipErrorNotSupported; }
}
