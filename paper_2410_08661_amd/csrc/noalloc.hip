// qeft_weak_grad_noalloc: the weak block's gradient for callers that can neither allocate device memory nor
// bring a workspace (code under HIP graph capture, tight serving or training loops, harnesses that forbid
// hipMalloc).  The partial slabs of the token split live in a file-scope device array instead of a caller's
// workspace; everything else is qeft_weak_grad's path (same kernels, same results bit for bit).
#include <atomic>

#include "qeft_internal.h"

using namespace qeft;

namespace {

constexpr size_t SCRATCH_BYTES = QEFT_NOALLOC_SCRATCH_BYTES;   // 14 MiB per GPU, held until the process ends

// The partial slabs.  In host code this name is only a handle for hipGetSymbolAddress: the memory is reached
// through the per-device address looked up below, never through the name.
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::atomic<void*> scratch_ptr[MAX_DEVICES];   // address of `scratch` on each device, looked up on first use there

// The array's address on the CURRENT device (every GPU has its own copy at its own address).
hipError_t scratch_on_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    void* p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        scratch_ptr[dev].store(p, std::memory_order_release);   // two threads racing here store the same address
    }
    *out = p;
    return hipSuccess;
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace

extern "C" int qeft_weak_grad_noalloc(const qeft_desc_t* desc, const void* dY, int64_t M, int64_t lddy, const void* Xw,
                                      int64_t ldxw, void* dW, int out_dtype, int accumulate, void* stream) {
    if (!desc) return QEFT_ERR_NULL;
    if (desc->bits != 3 && desc->bits != 4) return QEFT_ERR_BITS;
    const int oc = desc->out_features, k = desc->n_weak;
    if (oc <= 0 || desc->in_features <= 0 || desc->group_size <= 0 || k < 0 || k > desc->in_features || M < 0) return QEFT_ERR_SHAPE;
    if (out_dtype != QEFT_DTYPE_F16 && out_dtype != QEFT_DTYPE_F32) return QEFT_ERR_UNSUPPORTED;
    if (k == 0 || M == 0) return QEFT_OK;
    if (!dY || !Xw || !dW) return QEFT_ERR_NULL;
    if (lddy < oc || ldxw < k) return QEFT_ERR_SHAPE;
    if (!aligned16(dY) || !aligned16(Xw) || !aligned16(dW) || (lddy & 7) != 0 || (ldxw & 7) != 0) return QEFT_ERR_ALIGN;
    // only the tensor-core path has a scratch buffer to replace; other shapes go to qeft_weak_grad, which needs none for them
    if (!weak_grad_mfma_supported(oc, k, M)) return QEFT_ERR_UNSUPPORTED;
    const size_t need = weak_grad_mfma_workspace(oc, k, M);
    if (need > SCRATCH_BYTES) return QEFT_ERR_WORKSPACE;   // larger problems: qeft_weak_grad with a caller's workspace
    void* ptr = nullptr;
    if (scratch_on_current_device(&ptr) != hipSuccess) return QEFT_ERR_HIP;
    // nothing in the buffer has to start at zero: every slab entry the reduction reads is written by the strip kernel first
    return weak_grad_mfma(oc, k, (const __half*)dY, M, lddy, (const __half*)Xw, ldxw, dW, out_dtype == QEFT_DTYPE_F32,
                          accumulate != 0, ptr, (hipStream_t)stream) == hipSuccess
               ? QEFT_OK
               : QEFT_ERR_HIP;
}
