#include "qeft_internal.h"
namespace qeft {
bool gemv_supported(const Layer&, int64_t, int64_t) { return false; }
hipError_t gemv_fwd(const Layer&, const __half*, int64_t, int64_t, __half*, int64_t, hipStream_t) { return hipErrorNotSupported; }
}
