// Format conversion kernels: min-max round-to-nearest group quantization + bit packing
// (paper Sec. 3.1 for the three stored components; Sec. 6.1 / App. C for the quantizer),
// packing of externally chosen codes, and the inverse.  Integer results are bit-exact by
// construction: every float operation is a single correctly rounded IEEE fp32 operation.
// The __f*_rn functions of this toolchain are the plain operators, which the compiler would fuse
// (1 - i * step and p * hi - p * lo became fused multiply-adds and moved a scale across an fp16
// rounding tie in one group of three thousand), so this file is compiled with -ffp-contract=off
// (the build script passes it; a pragma here would not reach the header's inline functions).
#include <type_traits>

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

// Word wd of a row from the codes of its columns (code(j) is asked for j < Kq only).  Whole codes per word:
// columns per * wd .. + per - 1 at bits b i.  Dense 3-bit: every code whose bits 3j .. 3j+2 meet bits
// 32 wd .. 32 wd + 31 of the row, shifted to its place (the two codes at the ends may lie partly outside).
template <class F>
__device__ __forceinline__ uint32_t build_word(const Layer& L, int wd, F code) {
    uint32_t word = 0;
    if (L.dense) {
        const int j0 = (32 * wd) / 3, j1 = (32 * wd + 31) / 3;
        for (int j = j0; j <= j1; ++j) {
            if (j >= L.kq) break;
            const int sh = 3 * j - 32 * wd;   // -2 .. 31
            const uint32_t c = code(j);
            word |= sh >= 0 ? c << sh : c >> -sh;
        }
        return word;
    }
    const int per = (L.bits == 4) ? 8 : 10;
    for (int i = 0; i < per; ++i) {
        const int j = wd * per + i;
        if (j < L.kq) word |= code(j) << (L.bits * i);
    }
    return word;
}

// ---- step 2: one thread per 32-bit word: quantize its 8 / 10 columns and pack ------------
__global__ __launch_bounds__(256) void rtn_words_kernel(Layer L, const __half* __restrict__ W, int64_t ldw,
                                                        const __half* __restrict__ scales,
                                                        const __half* __restrict__ zeros, uint32_t* __restrict__ qweight) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)L.oc * L.stride) return;
    const int o = (int)(idx / L.stride), wd = (int)(idx % L.stride);
    const float qmax = (float)((1 << L.bits) - 1);
    qweight[idx] = build_word(L, wd, [&](int j) {
        const size_t gi = (size_t)o * L.gs + j / L.g;
        const float s = __half2float(scales[gi]);
        const float z = __half2float(zeros[gi]);
        const float v = __half2float(W[(size_t)o * ldw + j]);
        const float q = rintf(__fdiv_rn(v, s)) + z;
        return (uint32_t)fminf(fmaxf(q, 0.f), qmax);
    });
}

// ---- both steps in one pass for 4-bit codes and groups of 128 -----------------------------------
// One wavefront per (row, 512 columns = 4 groups = 64 words): lane l reads the 16 bytes of columns
// 8 l .. 8 l + 7 - its word - and belongs to group l / 16.  Minimum and maximum go through the 16
// lanes of the group with four data-parallel-primitive moves; every lane then derives the group's
// (scale, zero-point) with the same correctly rounded fp32 operations as the two-step kernels
// (bit-identical results), quantizes its 8 columns and stores its word: W is read once, with
// 16-byte loads, and the codes leave as 256 contiguous bytes per wavefront.  Columns past Kq count
// as zeros (neutral: a group's range always contains 0) and give zero codes; the wave of a row's
// last chunk also zeroes the row's padding parameters.
__device__ __forceinline__ float dpp16_min(float v) {
    auto mv = [](float x, auto ctrl) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value, 0xf, 0xf, false));
    };
    v = fminf(v, mv(v, std::integral_constant<int, 0xB1>{}));    // lane ^ 1
    v = fminf(v, mv(v, std::integral_constant<int, 0x4E>{}));    // lane ^ 2
    v = fminf(v, mv(v, std::integral_constant<int, 0x141>{}));   // mirrored halves of the row of 16
    v = fminf(v, mv(v, std::integral_constant<int, 0x140>{}));   // mirrored row
    return v;
}

__global__ __launch_bounds__(256) void rtn_fused_w4g128_kernel(Layer L, const __half* __restrict__ W, int64_t ldw,
                                                               uint32_t* __restrict__ qweight, __half* __restrict__ scales,
                                                               __half* __restrict__ zeros, int chunks) {
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    typedef _Float16 h8 __attribute__((ext_vector_type(8)));
    const int64_t wv = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (wv >= (int64_t)L.oc * chunks) return;
    const int o = (int)(wv / chunks), ch = (int)(wv % chunks);
    const int word = 64 * ch + lane, col = 8 * word;
    // Kq is a multiple of 8 here, so a word is entirely inside or entirely outside the row
    const bool live = col < L.kq;
    const u4 raw = live ? *reinterpret_cast<const u4*>(W + (size_t)o * ldw + col) : u4{0u, 0u, 0u, 0u};
    const h8 h = __builtin_bit_cast(h8, raw);
    float v[8], lo = 0.f, hi = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        v[e] = (float)h[e];
        lo = fminf(lo, v[e]);
        hi = fmaxf(hi, v[e]);
    }
    lo = dpp16_min(lo);
    hi = -dpp16_min(-hi);
    const float qmax = 15.f;
    const float s32 = __fdiv_rn(hi - lo, qmax);
    __half s16, z16;
    if (s32 == 0.f) {
        s16 = __float2half_rn(1.f);
        z16 = __float2half_rn(0.f);
    } else {
        s16 = __float2half_rn(s32);
        if (__half2float(s16) == 0.f) s16 = __ushort_as_half((unsigned short)1);  // smallest subnormal
        float z = rintf(__fdiv_rn(0.f - lo, __half2float(s16)));
        z = fminf(fmaxf(z, 0.f), qmax);
        z16 = __float2half_rn(z);
    }
    const float s = __half2float(s16), z = __half2float(z16);
    uint32_t out = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float q = rintf(__fdiv_rn(v[e], s)) + z;
        q = fminf(fmaxf(q, 0.f), qmax);
        out |= (uint32_t)q << (4 * e);
    }
    if (word < L.stride) qweight[(size_t)o * L.stride + word] = live ? out : 0u;
    const int gi = 4 * ch + (lane >> 4);
    if ((lane & 15) == 0 && gi < L.gs) {
        const bool real = gi < L.ng;
        scales[(size_t)o * L.gs + gi] = real ? s16 : __float2half_rn(0.f);
        zeros[(size_t)o * L.gs + gi] = real ? z16 : __float2half_rn(0.f);
    }
    // parameter padding past the groups this row's chunks cover
    if (ch == chunks - 1) {
        const int gi2 = 4 * chunks + lane;
        if (gi2 < L.gs) {
            scales[(size_t)o * L.gs + gi2] = __float2half_rn(0.f);
            zeros[(size_t)o * L.gs + gi2] = __float2half_rn(0.f);
        }
    }
}

// ---- group-wise grid search with truncation (paper Sec. 3.1) -------------------------------------
// For every (row, group): candidate i shrinks the min-max range (0 included) by p_i = 1 - i * step,
// derives (scale, zero-point) with the rules above, quantizes and scores the squared weight error;
// the first candidate with the smallest error is kept (candidate 0 = plain min-max).  One group per
// 16 lanes (a lane holds 8 consecutive columns; lanes past the group width hold zeros, which cost
// nothing), four groups per wavefront.  Every operation is a single correctly rounded fp32
// operation (the intrinsics keep the compiler from fusing multiply and add) and the error is
// summed in a fixed order - a lane's 8 columns left to right, then a balanced tree over the 16
// lanes - so that the decisions can be reproduced exactly elsewhere.
__device__ __forceinline__ float dpp16_sum(float v) {
    auto mv = [](float x, auto ctrl) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value, 0xf, 0xf, false));
    };
    v = __fadd_rn(v, mv(v, std::integral_constant<int, 0xB1>{}));
    v = __fadd_rn(v, mv(v, std::integral_constant<int, 0x4E>{}));
    v = __fadd_rn(v, mv(v, std::integral_constant<int, 0x141>{}));
    v = __fadd_rn(v, mv(v, std::integral_constant<int, 0x140>{}));
    return v;
}

__global__ __launch_bounds__(256) void search_params_kernel(Layer L, const __half* __restrict__ W, int64_t ldw,
                                                            __half* __restrict__ scales, __half* __restrict__ zeros,
                                                            int chunks, int n_grid, float step) {
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    typedef _Float16 h8 __attribute__((ext_vector_type(8)));
    const int64_t wv = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (wv >= (int64_t)L.oc * chunks) return;
    const int o = (int)(wv / chunks), ch = (int)(wv % chunks);
    const int grp = 4 * ch + (lane >> 4), t = lane & 15;   // grp < gs: chunks = gs / 4
    const int col = grp * L.g + 8 * t;
    const bool live = grp < L.ng && 8 * t < L.g && col < L.kq;   // Kq % 8 == 0: whole octets
    const u4 raw = live ? *reinterpret_cast<const u4*>(W + (size_t)o * ldw + col) : u4{0u, 0u, 0u, 0u};
    const h8 h = __builtin_bit_cast(h8, raw);
    float v[8], lo0 = 0.f, hi0 = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        v[e] = (float)h[e];
        lo0 = fminf(lo0, v[e]);
        hi0 = fmaxf(hi0, v[e]);
    }
    lo0 = dpp16_min(lo0);
    hi0 = -dpp16_min(-hi0);
    const float qmax = (float)((1 << L.bits) - 1);
    float best_e = __builtin_inff();
    __half best_s = __float2half_rn(1.f), best_z = __float2half_rn(0.f);
    for (int i = 0; i < n_grid; ++i) {
        const float p = __fsub_rn(1.f, __fmul_rn((float)i, step));
        const float lo = __fmul_rn(p, lo0), hi = __fmul_rn(p, hi0);
        const float s32 = __fdiv_rn(__fsub_rn(hi, lo), qmax);
        __half s16, z16;
        if (s32 == 0.f) {
            s16 = __float2half_rn(1.f);
            z16 = __float2half_rn(0.f);
        } else {
            s16 = __float2half_rn(s32);
            if (__half2float(s16) == 0.f) s16 = __ushort_as_half((unsigned short)1);
            float z = rintf(__fdiv_rn(__fsub_rn(0.f, lo), __half2float(s16)));
            z = fminf(fmaxf(z, 0.f), qmax);
            z16 = __float2half_rn(z);
        }
        const float s = __half2float(s16), z = __half2float(z16);
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float q = __fadd_rn(rintf(__fdiv_rn(v[e], s)), z);
            q = fminf(fmaxf(q, 0.f), qmax);
            const float d = __fsub_rn(v[e], __fmul_rn(s, __fsub_rn(q, z)));
            acc = __fadd_rn(acc, __fmul_rn(d, d));
        }
        const float err = dpp16_sum(acc);
        if (err < best_e) {
            best_e = err;
            best_s = s16;
            best_z = z16;
        }
    }
    if (t == 0) {
        const bool real = grp < L.ng;
        scales[(size_t)o * L.gs + grp] = real ? best_s : __float2half_rn(0.f);
        zeros[(size_t)o * L.gs + grp] = real ? best_z : __float2half_rn(0.f);
    }
}

__global__ __launch_bounds__(256) void pack_words_kernel(Layer L, const uint8_t* __restrict__ codes,
                                                         uint32_t* __restrict__ qweight) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)L.oc * L.stride) return;
    const int o = (int)(idx / L.stride), wd = (int)(idx % L.stride);
    const uint32_t mask = (1u << L.bits) - 1u;
    qweight[idx] = build_word(L, wd, [&](int j) { return (uint32_t)codes[(size_t)o * L.kq + j] & mask; });
}

__global__ __launch_bounds__(256) void unpack_codes_kernel(Layer L, uint8_t* __restrict__ codes) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)L.oc * L.kq) return;
    const int o = (int)(idx / L.kq), j = (int)(idx % L.kq);
    codes[idx] = (uint8_t)code_at(L, L.qweight + (size_t)o * L.stride, j);
}

// One thread per 8 columns of a row of the mixed weight: 16 bytes out.
__global__ __launch_bounds__(256) void dequantize_kernel(Layer L, __half* __restrict__ out) {
    const int chunks = L.ic >> 3;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)L.oc * chunks) return;
    const int o = (int)(idx / chunks), j0 = 8 * (int)(idx % chunks);
    const uint32_t* row = L.qweight + (size_t)o * L.stride;
    __half v[8];
    if (j0 + 8 <= L.kq && (L.g & 7) == 0) {   // the usual case: eight quantized columns of one group
        const size_t gi = (size_t)o * L.gs + j0 / L.g;
        const float sc = __half2float(L.scales[gi]), zp = __half2float(L.zeros[gi]);
        if (L.dense) {                        // 24 bits starting at bit 3 j0 = 24 (j0 / 8) of the row
            const int bit = 3 * j0, w0 = bit >> 5, sh = bit & 31;
            uint32_t c = row[w0] >> sh;
            if (sh > 8) c |= row[w0 + 1] << (32 - sh);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = __float2half_rn(sc * ((float)((c >> (3 * e)) & 7u) - zp));
        } else if (L.bits == 4) {
            const uint32_t c = row[j0 >> 3];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = __float2half_rn(sc * ((float)((c >> (4 * e)) & 15u) - zp));
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = __float2half_rn(sc * ((float)code_at(L, row, j0 + e) - zp));
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int j = j0 + e;
            if (j < L.kq) {
                const size_t gi = (size_t)o * L.gs + j / L.g;
                v[e] = __float2half_rn(__half2float(L.scales[gi]) * ((float)code_at(L, row, j) - __half2float(L.zeros[gi])));
            } else {
                v[e] = L.weak[(size_t)o * L.k + (j - L.kq)];
            }
        }
    }
    *reinterpret_cast<uint4*>(out + (size_t)o * L.ic + j0) = *reinterpret_cast<const uint4*>(v);
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
    if (L.kq > 0 && L.bits == 4 && L.g == 128 && (L.kq & 7) == 0 && (ldw & 7) == 0 && ((uintptr_t)W & 15) == 0) {
        const int chunks = ceil_div(L.stride, 64);
        rtn_fused_w4g128_kernel<<<ceil_div((int64_t)L.oc * chunks, 4), 256, 0, s>>>(L, W, ldw, qweight, scales, zeros, chunks);
    } else if (L.kq > 0) {
        const int64_t pairs = (int64_t)L.oc * L.gs;
        rtn_params_kernel<<<ceil_div(pairs, 4), 256, 0, s>>>(L, W, ldw, scales, zeros);
        rtn_words_kernel<<<ceil_div((int64_t)L.oc * L.stride, 256), 256, 0, s>>>(L, W, ldw, scales, zeros, qweight);
    }
    copy2d(W + L.kq, ldw, weak, L.k, L.oc, L.k, s);
    return hipGetLastError();
}

bool pack_search_supported(const Layer& L, int64_t ldw, const void* W) {
    return (L.g & 7) == 0 && L.g <= 128 && (L.kq & 7) == 0 && (ldw & 7) == 0 && ((uintptr_t)W & 15) == 0;
}

hipError_t pack_search(const Layer& L, const __half* W, int64_t ldw, int n_grid, float step, uint32_t* qweight,
                       __half* scales, __half* zeros, __half* weak, hipStream_t s) {
    if (L.kq > 0) {
        const int chunks = L.gs / 4;
        search_params_kernel<<<ceil_div((int64_t)L.oc * chunks, 4), 256, 0, s>>>(L, W, ldw, scales, zeros, chunks, n_grid, step);
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

hipError_t dequantize_fp16(const Layer& L, __half* out, hipStream_t s) {
    const int64_t n = (int64_t)L.oc * (L.ic >> 3);
    dequantize_kernel<<<ceil_div(n, 256), 256, 0, s>>>(L, out);
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
