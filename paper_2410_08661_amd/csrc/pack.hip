// Format conversion kernels: min-max round-to-nearest group quantization + bit packing
// (paper Sec. 3.1 for the three stored components; Sec. 6.1 / App. C for the quantizer),
// packing of externally chosen codes, and the inverse.  Integer results are bit-exact by
// construction: every float operation is a single correctly rounded IEEE fp32 operation
// (explicit __fdiv_rn / rintf, no contraction possible).
#include "qeft_internal.h"

namespace qeft {
namespace {

// ---- step 1: (scale, zero) of every (row, group); one wavefront per pair ------------------
__global__ __launch_bounds__(256) void rtn_params_kernel(Layer L, const __half* __restrict__ W, int64_t ldw,
                                                         __half* __restrict__ scales, __half* __restrict__ zeros) {
    const int64_t pair = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);   // over [OC][group_stride]
    const int lane = threadIdx.x & 63;
    if (pair >= (int64_t)L.oc * L.gs) return;
    const int o = (int)(pair / L.gs), gi = (int)(pair % L.gs);
    if (gi >= L.ng) {   // padding entry
        if (lane == 0) {
            scales[pair] = __float2half_rn(0.f);
            zeros[pair] = __float2half_rn(0.f);
        }
        return;
    }
    const int j0 = gi * L.g;
    const int len = min(L.g, L.kq - j0);
    float lo = 0.f, hi = 0.f;  // the range always contains 0
    for (int j = lane; j < len; j += 64) {
        const float v = __half2float(W[(size_t)o * ldw + j0 + j]);
        lo = fminf(lo, v);
        hi = fmaxf(hi, v);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, off, 64));
        hi = fmaxf(hi, __shfl_xor(hi, off, 64));
    }
    if (lane == 0) {
        const float qmax = (float)((1 << L.bits) - 1);
        const float s32 = __fdiv_rn(hi - lo, qmax);
        __half s16, z16;
        if (s32 == 0.f) {
            s16 = __float2half_rn(1.f);
            z16 = __float2half_rn(0.f);
        } else {
            s16 = __float2half_rn(s32);
            if (__half2float(s16) == 0.f) s16 = __ushort_as_half((unsigned short)1);  // smallest subnormal
            const float s = __half2float(s16);
            float z = rintf(__fdiv_rn(0.f - lo, s));
            z = fminf(fmaxf(z, 0.f), qmax);
            z16 = __float2half_rn(z);
        }
        scales[pair] = s16;
        zeros[pair] = z16;
    }
}

// ---- step 2: one thread per 32-bit word: quantize its 8 / 10 columns and pack ------------
__global__ __launch_bounds__(256) void rtn_words_kernel(Layer L, const __half* __restrict__ W, int64_t ldw,
                                                        const __half* __restrict__ scales,
                                                        const __half* __restrict__ zeros, uint32_t* __restrict__ qweight) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)L.oc * L.stride) return;
    const int o = (int)(idx / L.stride), wd = (int)(idx % L.stride);
    const int per = (L.bits == 4) ? 8 : 10;
    const float qmax = (float)((1 << L.bits) - 1);
    uint32_t word = 0;
    for (int i = 0; i < per; ++i) {
        const int j = wd * per + i;
        if (j < L.kq) {
            const size_t gi = (size_t)o * L.gs + j / L.g;
            const float s = __half2float(scales[gi]);
            const float z = __half2float(zeros[gi]);
            const float v = __half2float(W[(size_t)o * ldw + j]);
            float q = rintf(__fdiv_rn(v, s)) + z;
            q = fminf(fmaxf(q, 0.f), qmax);
            word |= (uint32_t)q << (L.bits * i);
        }
    }
    qweight[idx] = word;
}

__global__ __launch_bounds__(256) void pack_words_kernel(Layer L, const uint8_t* __restrict__ codes,
                                                         uint32_t* __restrict__ qweight) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)L.oc * L.stride) return;
    const int o = (int)(idx / L.stride), wd = (int)(idx % L.stride);
    const int per = (L.bits == 4) ? 8 : 10;
    const uint32_t mask = (1u << L.bits) - 1u;
    uint32_t word = 0;
    for (int i = 0; i < per; ++i) {
        const int j = wd * per + i;
        if (j < L.kq) word |= ((uint32_t)codes[(size_t)o * L.kq + j] & mask) << (L.bits * i);
    }
    qweight[idx] = word;
}

__global__ __launch_bounds__(256) void unpack_codes_kernel(Layer L, uint8_t* __restrict__ codes) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)L.oc * L.kq) return;
    const int o = (int)(idx / L.kq), j = (int)(idx % L.kq);
    const int per = (L.bits == 4) ? 8 : 10;
    const uint32_t word = L.qweight[(size_t)o * L.stride + j / per];
    codes[idx] = (uint8_t)((word >> (L.bits * (j % per))) & ((1u << L.bits) - 1u));
}

// compact [OC][G] parameters into the padded [OC][group_stride] arrays (padding zero)
__global__ __launch_bounds__(256) void pad_groups_kernel(Layer L, const __half* __restrict__ s_in,
                                                         const __half* __restrict__ z_in, __half* __restrict__ s_out,
                                                         __half* __restrict__ z_out) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)L.oc * L.gs) return;
    const int o = (int)(idx / L.gs), gi = (int)(idx % L.gs);
    const bool real = gi < L.ng;
    s_out[idx] = real ? s_in[(size_t)o * L.ng + gi] : __float2half_rn(0.f);
    z_out[idx] = real ? z_in[(size_t)o * L.ng + gi] : __float2half_rn(0.f);
}

// rows x cols fp16 copy between two leading dimensions
__global__ __launch_bounds__(256) void copy2d_kernel(const __half* __restrict__ src, int64_t lds, __half* __restrict__ dst,
                                                     int64_t ldd, int64_t rows, int cols) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= rows * cols) return;
    const int64_t r = idx / cols;
    const int c = (int)(idx % cols);
    dst[r * ldd + c] = src[r * lds + c];
}

void copy2d(const __half* src, int64_t lds, __half* dst, int64_t ldd, int64_t rows, int cols, hipStream_t s) {
    if (rows * cols == 0 || src == dst) return;
    copy2d_kernel<<<ceil_div(rows * cols, 256), 256, 0, s>>>(src, lds, dst, ldd, rows, cols);
}

}  // namespace

hipError_t pack_rtn(const Layer& L, const __half* W, int64_t ldw, uint32_t* qweight, __half* scales, __half* zeros,
                    __half* weak, hipStream_t s) {
    if (L.kq > 0) {
        const int64_t pairs = (int64_t)L.oc * L.gs;
        rtn_params_kernel<<<ceil_div(pairs, 4), 256, 0, s>>>(L, W, ldw, scales, zeros);
        rtn_words_kernel<<<ceil_div((int64_t)L.oc * L.stride, 256), 256, 0, s>>>(L, W, ldw, scales, zeros, qweight);
    }
    copy2d(W + L.kq, ldw, weak, L.k, L.oc, L.k, s);
    return hipGetLastError();
}

hipError_t pack_codes(const Layer& L, const uint8_t* codes, const __half* scales_in, const __half* zeros_in,
                      const __half* weak_in, uint32_t* qweight, __half* scales, __half* zeros, __half* weak, hipStream_t s) {
    if (L.kq > 0) {
        pack_words_kernel<<<ceil_div((int64_t)L.oc * L.stride, 256), 256, 0, s>>>(L, codes, qweight);
        pad_groups_kernel<<<ceil_div((int64_t)L.oc * L.gs, 256), 256, 0, s>>>(L, scales_in, zeros_in, scales, zeros);
    }
    copy2d(weak_in, L.k, weak, L.k, L.oc, L.k, s);
    return hipGetLastError();
}

hipError_t unpack(const Layer& L, uint8_t* codes, __half* scales, __half* zeros, __half* weak, hipStream_t s) {
    if (L.kq > 0) {
        if (codes) unpack_codes_kernel<<<ceil_div((int64_t)L.oc * L.kq, 256), 256, 0, s>>>(L, codes);
        if (scales) copy2d(L.scales, L.gs, scales, L.ng, L.oc, L.ng, s);
        if (zeros) copy2d(L.zeros, L.gs, zeros, L.ng, L.oc, L.ng, s);
    }
    if (weak) copy2d(L.weak, L.k, weak, L.k, L.oc, L.k, s);
    return hipGetLastError();
}

}  // namespace qeft
