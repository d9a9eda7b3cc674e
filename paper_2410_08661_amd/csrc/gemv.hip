// Decode path (paper Sec. 3.2.1): Y = X . W^T for M <= 16 rows in one fused pass over the
// packed 4-bit codes, the group parameters and the fp16 weak block.  HBM-bound: the kernel
// streams every stored byte exactly once with 128-bit loads.
//
// Mapping.  The product runs on the 16x16x32 fp16 MFMA with the M (<= 16, zero padded)
// activation rows as the A operand and 16 output channels as the B operand.  In that
// instruction lane l supplies 8 contraction elements of row/column l % 16 for the slot
// l / 16, and one packed 32-bit word holds exactly 8 codes: a lane's 128-bit load (4 words
// = 32 codes) therefore feeds 4 MFMAs with no cross-lane movement, and the 4 slots of a
// load cover 128 consecutive columns = one quantization group.  Which column a contraction
// slot stands for is free as long as A and B agree, so the activations are permuted to the
// order the nibbles come out of the mask-and-or conversion (pairs (0,4) (1,5) (2,6) (3,7)).
//
// Dequantization never touches the weights: the codes enter the MFMA as the exact fp16
// numbers 1024 + q (exponent bits or-ed onto the nibble), one extra MFMA against a vector of
// ones gives Sx = sum of the group's activations, and the group's contribution is
//     s * (sum x*(1024+q) - (1024 + z) * Sx) = s * sum x*(q - z)
// applied to the 16x16 fp32 accumulator: 2 FMAs per 32 weights and lane, any fp16 zero-point.
// The weak block is a plain fp16 B operand accumulated into the same tile.
// The K range is split over the waves of a workgroup (step s -> wave s % KS) and reduced
// through LDS in a fixed order: no atomics, run-to-run deterministic.
#include "qeft_internal.h"
#include <cstdlib>

namespace qeft {
namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ h8 as_h8(u4 v) { return __builtin_bit_cast(h8, v); }

__device__ __forceinline__ u4 load16(const void* p) { return *reinterpret_cast<const u4*>(p); }

// 8 codes of one word as fp16 (1024 + q), in slot order (0,4)(1,5)(2,6)(3,7)
__device__ __forceinline__ h8 codes_to_h8(uint32_t w) {
    u4 r;
    r.x = (w & 0x000f000fu) | 0x64006400u;
    r.y = ((w >> 4) & 0x000f000fu) | 0x64006400u;
    r.z = ((w >> 8) & 0x000f000fu) | 0x64006400u;
    r.w = ((w >> 12) & 0x000f000fu) | 0x64006400u;
    return as_h8(r);
}

// 8 consecutive activations (x0..x7 in 4 registers) to the same slot order
__device__ __forceinline__ h8 permute_x(u4 v) {
    u4 r;
    r.x = __builtin_amdgcn_perm(v.z, v.x, 0x05040100u);  // (x0, x4)
    r.y = __builtin_amdgcn_perm(v.z, v.x, 0x07060302u);  // (x1, x5)
    r.z = __builtin_amdgcn_perm(v.w, v.y, 0x05040100u);  // (x2, x6)
    r.w = __builtin_amdgcn_perm(v.w, v.y, 0x07060302u);  // (x3, x7)
    return as_h8(r);
}

constexpr int PF = 4;  // K steps whose loads are issued together

template <int R>
__global__ __launch_bounds__(256) void gemv_w4_kernel(Layer L, const __half* __restrict__ X, int M, int64_t ldx,
                                                      __half* __restrict__ Y, int64_t ldy) {
    extern __shared__ float red[];  // [KS-1][R][4][64]
    // The wave index is made provably wave-uniform: every branch on the K step must be a
    // scalar branch, because MFMA executes whatever the EXEC mask says.
    const int lane = threadIdx.x & 63, KS = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, kb = lane >> 4;
    const int row0 = blockIdx.x * (16 * R);
    const int nq = L.ng;                       // quantized steps: one group of 128 columns each
    const int nsteps = nq + (L.k + 31) / 32;   // + weak steps of 32 columns each

    const uint32_t* wrow[R];
    const __half* srow[R];
    const __half* zrow[R];
    const __half* krow[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int o = min(row0 + 16 * r + n, L.oc - 1);
        wrow[r] = L.qweight + (size_t)o * L.stride;
        srow[r] = L.scales + (size_t)o * L.ng;
        zrow[r] = L.zeros + (size_t)o * L.ng;
        krow[r] = L.weak + (size_t)o * L.k;
    }
    const bool mvalid = n < M;                 // this lane's activation row exists
    const __half* xrow = X + (size_t)(mvalid ? n : 0) * ldx;

    f4 y[R];
#pragma unroll
    for (int r = 0; r < R; ++r) y[r] = f4{0.f, 0.f, 0.f, 0.f};
    const u4 zero4 = u4{0u, 0u, 0u, 0u};
    u4 ones4 = u4{0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
    const h8 ones = as_h8(ones4);

    for (int s0 = wave; s0 < nsteps; s0 += KS * PF) {
        u4 wq[PF][R];
        u4 xa[PF][4];
        float sc[PF][R], zc[PF][R];
        // ---- issue every load of this chunk ------------------------------------------------
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const int s = s0 + p * KS;
            if (s < nq) {
                const int word = 4 * (4 * s + kb);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    wq[p][r] = (word < L.stride) ? load16(wrow[r] + word) : zero4;
                    sc[p][r] = __half2float(srow[r][s]);
                    zc[p][r] = __half2float(zrow[r][s]);
                }
                const int col = 128 * s + 32 * kb;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    xa[p][i] = (mvalid && col + 8 * i < L.kq) ? load16(xrow + col + 8 * i) : zero4;
            } else if (s < nsteps) {
                const int c0 = 32 * (s - nq) + 8 * kb;
#pragma unroll
                for (int r = 0; r < R; ++r) wq[p][r] = (c0 < L.k) ? load16(krow[r] + c0) : zero4;
                xa[p][0] = (mvalid && c0 < L.k) ? load16(xrow + L.kq + c0) : zero4;
            }
        }
        // ---- consume ----------------------------------------------------------------------
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const int s = s0 + p * KS;
            if (s < nq) {
                h8 a[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) a[i] = permute_x(xa[p][i]);
                f4 sx = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int i = 0; i < 4; ++i) sx = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[i], ones, sx, 0, 0, 0);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    f4 acc = f4{0.f, 0.f, 0.f, 0.f};
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[0], codes_to_h8(wq[p][r].x), acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[1], codes_to_h8(wq[p][r].y), acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[2], codes_to_h8(wq[p][r].z), acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[3], codes_to_h8(wq[p][r].w), acc, 0, 0, 0);
                    const float c = 1024.f + zc[p][r];
                    const float sf = sc[p][r];
#pragma unroll
                    for (int e = 0; e < 4; ++e) y[r][e] = fmaf(sf, fmaf(-c, sx[e], acc[e]), y[r][e]);
                }
            } else if (s < nsteps) {
                const h8 a = as_h8(xa[p][0]);
#pragma unroll
                for (int r = 0; r < R; ++r) y[r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, as_h8(wq[p][r]), y[r], 0, 0, 0);
            }
        }
    }

    // ---- reduce the K split: waves 1..KS-1 hand their tiles to wave 0 through LDS ---------------
    if (wave > 0) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < 4; ++e) red[(((wave - 1) * R + r) * 4 + e) * 64 + lane] = y[r][e];
    }
    __syncthreads();
    if (wave == 0) {
        for (int w = 1; w < KS; ++w)
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int e = 0; e < 4; ++e) y[r][e] += red[(((w - 1) * R + r) * 4 + e) * 64 + lane];
        // accumulator element e of lane l is row 4*(l/16)+e, column l%16 of the 16x16 tile
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int o = row0 + 16 * r + n;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int m = 4 * kb + e;
                if (m < M && o < L.oc) Y[(size_t)m * ldy + o] = __float2half_rn(y[r][e]);
            }
        }
    }
}

}  // namespace

bool gemv_supported(const Layer& L, int64_t M, int64_t ldx) {
    (void)ldx;
    return M >= 1 && L.bits == 4 && L.g == 128 && (L.kq % 8) == 0 && (L.k % 8) == 0;
}

hipError_t gemv_fwd(const Layer& L, const __half* X, int64_t M, int64_t ldx, __half* Y, int64_t ldy, hipStream_t s) {
    constexpr int R = 1;
    const char* e = getenv("QEFT_DBG_KS");
    const int ks = e ? atoi(e) : 4;
    const int grid = ceil_div(L.oc, 16 * R);
    const size_t lds = (size_t)(ks - 1) * R * 4 * 64 * sizeof(float);
    gemv_w4_kernel<R><<<grid, 64 * ks, lds, s>>>(L, X, (int)M, ldx, Y, ldy);
    return hipGetLastError();
}

}  // namespace qeft
