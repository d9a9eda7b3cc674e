// Generic kernels: correct for every shape, bit width and alignment the format allows.
// They are the fallback for shapes the tiled kernels do not cover (odd k, odd group
// sizes, 3-bit backward); plain loops, fp32 accumulation, no tiling.
#include "qeft_internal.h"

namespace qeft {
namespace {

constexpr int MB = 8;  // rows of X / dY handled per thread block

// One element of the mixed weight (Sec. 3.1): s * (q - z) for j < Kq, the fp16 weak block otherwise.
__device__ __forceinline__ float weight_at(const Layer& L, int o, int j) {
    if (j >= L.kq) return __half2float(L.weak[(size_t)o * L.k + (j - L.kq)]);
    const uint32_t code = code_at(L, L.qweight + (size_t)o * L.stride, j);
    const size_t gi = (size_t)o * L.gs + j / L.g;
    return __half2float(L.scales[gi]) * ((float)code - __half2float(L.zeros[gi]));
}

__global__ __launch_bounds__(256) void fwd_generic_kernel(Layer L, const __half* __restrict__ X, int M, int64_t ldx,
                                                          __half* __restrict__ Y, int64_t ldy) {
    const int o = blockIdx.x;
    const int m0 = blockIdx.y * MB;
    const int nm = min(MB, M - m0);
    float acc[MB];
#pragma unroll
    for (int i = 0; i < MB; ++i) acc[i] = 0.f;
    for (int j = threadIdx.x; j < L.ic; j += 256) {
        const float w = weight_at(L, o, j);
#pragma unroll
        for (int i = 0; i < MB; ++i)
            if (i < nm) acc[i] += __half2float(X[(size_t)(m0 + i) * ldx + j]) * w;
    }
    __shared__ float red[MB][256];
#pragma unroll
    for (int i = 0; i < MB; ++i) red[i][threadIdx.x] = acc[i];
    __syncthreads();
    for (int sft = 128; sft > 0; sft >>= 1) {
        if ((int)threadIdx.x < sft) {
#pragma unroll
            for (int i = 0; i < MB; ++i) red[i][threadIdx.x] += red[i][threadIdx.x + sft];
        }
        __syncthreads();
    }
    if ((int)threadIdx.x < nm) Y[(size_t)(m0 + threadIdx.x) * ldy + o] = __float2half_rn(red[threadIdx.x][0]);
}

__global__ __launch_bounds__(256) void dx_generic_kernel(Layer L, const __half* __restrict__ dY, int M, int64_t lddy,
                                                         __half* __restrict__ dX, int64_t lddx) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    const int m0 = blockIdx.y * MB;
    const int nm = min(MB, M - m0);
    if (c >= L.ic) return;
    float acc[MB];
#pragma unroll
    for (int i = 0; i < MB; ++i) acc[i] = 0.f;
    for (int o = 0; o < L.oc; ++o) {
        const float w = weight_at(L, o, c);
#pragma unroll
        for (int i = 0; i < MB; ++i)
            if (i < nm) acc[i] += __half2float(dY[(size_t)(m0 + i) * lddy + o]) * w;
    }
#pragma unroll
    for (int i = 0; i < MB; ++i)
        if (i < nm) dX[(size_t)(m0 + i) * lddx + c] = __float2half_rn(acc[i]);
}

__global__ __launch_bounds__(256) void weak_grad_generic_kernel(int oc, int k, const __half* __restrict__ dY, int M,
                                                                int64_t lddy, const __half* __restrict__ Xw, int64_t ldxw,
                                                                void* dW, int out_f32, int accumulate) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)oc * k) return;
    const int o = (int)(idx / k), c = (int)(idx % k);
    float acc = 0.f;
    for (int m = 0; m < M; ++m) acc += __half2float(dY[(size_t)m * lddy + o]) * __half2float(Xw[(size_t)m * ldxw + c]);
    if (out_f32) {
        float* p = (float*)dW + idx;
        *p = accumulate ? *p + acc : acc;
    } else {
        __half* p = (__half*)dW + idx;
        *p = __float2half_rn(accumulate ? __half2float(*p) + acc : acc);
    }
}

}  // namespace

hipError_t fwd_generic(const Layer& L, const __half* X, int64_t M, int64_t ldx, __half* Y, int64_t ldy, hipStream_t s) {
    for (int64_t m0 = 0; m0 < M; m0 += 65535LL * MB) {   // grid.y limit
        const int mm = (int)((M - m0 < 65535LL * MB) ? (M - m0) : 65535LL * MB);
        dim3 grid(L.oc, ceil_div(mm, MB));
        fwd_generic_kernel<<<grid, 256, 0, s>>>(L, X + m0 * ldx, mm, ldx, Y + m0 * ldy, ldy);
    }
    return hipGetLastError();
}

hipError_t bwd_dx_generic(const Layer& L, const __half* dY, int64_t M, int64_t lddy, __half* dX, int64_t lddx,
                          hipStream_t s) {
    for (int64_t m0 = 0; m0 < M; m0 += 65535LL * MB) {
        const int mm = (int)((M - m0 < 65535LL * MB) ? (M - m0) : 65535LL * MB);
        dim3 grid(ceil_div(L.ic, 256), ceil_div(mm, MB));
        dx_generic_kernel<<<grid, 256, 0, s>>>(L, dY + m0 * lddy, mm, lddy, dX + m0 * lddx, lddx);
    }
    return hipGetLastError();
}

hipError_t weak_grad_generic(int oc, int k, const __half* dY, int64_t M, int64_t lddy, const __half* Xw, int64_t ldxw,
                             void* dW, int out_f32, int accumulate, hipStream_t s) {
    const int64_t n = (int64_t)oc * k;
    if (n == 0) return hipSuccess;
    weak_grad_generic_kernel<<<ceil_div(n, 256), 256, 0, s>>>(oc, k, dY, (int)M, lddy, Xw, ldxw, dW, out_f32, accumulate);
    return hipGetLastError();
}

}  // namespace qeft
