// Prefill / fine-tune path (paper Sec. 3.3): the large-M products of the fused layer as tiled
// fp16 MFMA GEMMs with fp32 accumulation.
//
//   forward   Y [M][OC]  = X  . W^T        contraction over IC  (quantized part + weak block)
//   backward  dX[M][IC]  = dY . W          contraction over OC  (through the full mixed weight)
//
// Both are computed "transposed": the weight side is the MFMA A operand (rows = OC for the
// forward), the activation side the B operand (columns = tokens).  With the 32x32x16 MFMA a
// lane then owns 4 consecutive output channels of one token, i.e. 8 contiguous bytes of the
// row-major result, so the epilogue stores straight from the accumulators.
//
// Tiling: a workgroup of 4 waves (2 x 2) owns a 256 x 256 output tile, each wave 128 x 128
// (4 x 4 MFMA tiles, 256 accumulator registers).  K advances in stages of 64: both operand
// tiles (256 rows x 64 halfs, rows of 128 bytes, 16-byte chunks XOR-swizzled by the row so
// fragment reads are conflict-free) are double-buffered in LDS, 128 KB of the CU's 160 KB.
// The next stage's global loads are issued before the current stage's MFMAs; the weights
// are dequantized in registers on their way into LDS, so the MFMA loop sees plain fp16.
//
// Dequantization: codes become the exact fp16 numbers 1024 + q by or-ing exponent bits onto
// the masked nibbles (two codes per instruction); then ((1024+q) - 1024 - z) * s in packed
// fp16: the two subtractions keep any fp16 zero-point exact up to one rounding.  The nibbles
// of a word come out in the order (0,4)(1,5)(2,6)(3,7); the activations of quantized stages
// are permuted to the same order when they are written to LDS.
#include "qeft_internal.h"

namespace qeft {
namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));

constexpr int BT = 256;                 // tile rows of either operand
constexpr int BK = 64;                  // K per stage
constexpr int TILE_BYTES = BT * BK * 2; // 32 KB
constexpr int GEMM_LDS = 4 * TILE_BYTES;

__device__ __forceinline__ u4 ld16(const void* p) { return *reinterpret_cast<const u4*>(p); }
__device__ __forceinline__ h8 as_h8(u4 v) { return __builtin_bit_cast(h8, v); }
__device__ __forceinline__ uint32_t h2_bits(h2 v) { return __builtin_bit_cast(uint32_t, v); }
__device__ __forceinline__ h2 bits_h2(uint32_t v) { return __builtin_bit_cast(h2, v); }

// byte offset of 16-byte chunk `c` (0..7) of row `r` inside a 256 x 64 half tile
__device__ __forceinline__ int tile_off(int r, int c) { return r * 128 + ((c ^ (r & 7)) << 4); }

struct Consts {
    uint32_t mask, magic;
};
__device__ __forceinline__ Consts make_consts() {
    Consts c{0x000f000fu, 0x64006400u};
    asm volatile("" : "+v"(c.mask), "+v"(c.magic));  // opaque: (w & mask) | magic selects v_and_or_b32
    return c;
}

// 8 activations x0..x7 -> (x0,x4)(x1,x5)(x2,x6)(x3,x7)
__device__ __forceinline__ u4 permute_x(u4 v) {
    u4 r;
    r.x = __builtin_amdgcn_perm(v.z, v.x, 0x05040100u);
    r.y = __builtin_amdgcn_perm(v.z, v.x, 0x07060302u);
    r.z = __builtin_amdgcn_perm(v.w, v.y, 0x05040100u);
    r.w = __builtin_amdgcn_perm(v.w, v.y, 0x07060302u);
    return r;
}

// one word of 8 codes -> 8 dequantized fp16 weights in nibble order.  nz = (-1024 - z ... ) is
// applied as two exact/rounded steps: (h - 1024) is exact, (.. - z) rounds once, (.. * s) once.
__device__ __forceinline__ u4 dequant_word(uint32_t w, h2 z2, h2 s2, Consts c) {
    const h2 k1024 = h2{(_Float16)1024.f, (_Float16)1024.f};
    u4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const h2 h = bits_h2(((w >> (4 * i)) & c.mask) | c.magic);
        r[i] = h2_bits(((h - k1024) - z2) * s2);
    }
    return r;
}

// ---- forward -----------------------------------------------------------------------------------------
// Raw global data of one stage, held in registers until the previous stage's MFMAs are issued.
struct FwdStage {
    u4 a[8];        // quantized stage: a[0], a[1] = 4 code words of rows r0 and r0+128; weak stage: 8 fp16 chunks
    u4 b[8];        // 8 chunks of X
    uint32_t sz[2]; // (scale, zero) halfs of the two rows
};

__global__ __launch_bounds__(256) void gemm_fwd_kernel(Layer L, const __half* __restrict__ X, int M, int64_t ldx,
                                                       __half* __restrict__ Y, int64_t ldy, int tiles_oc) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;   // wave position: OC half, token half
    // consecutive workgroups walk the OC tiles of one token panel: the panel of X stays in L2
    const int t_oc = blockIdx.x % tiles_oc, t_m = blockIdx.x / tiles_oc;
    const int oc0 = t_oc * BT, m0 = t_m * BT;
    const int nq_st = (L.kq + BK - 1) / BK, nw_st = (L.k + BK - 1) / BK, nst = nq_st + nw_st;
    const Consts cst = make_consts();
    const u4 zero4 = u4{0u, 0u, 0u, 0u};

    // producer coordinates
    const int ar = tid >> 1, ah = tid & 1;               // quantized A: rows ar, ar+128; half ah of the stage
    const int arow0 = min(oc0 + ar, L.oc - 1), arow1 = min(oc0 + ar + 128, L.oc - 1);

    auto load_stage = [&](FwdStage& s, int st) {
        if (st < nq_st) {
            s.a[0] = ld16(L.qweight + (size_t)arow0 * L.stride + 8 * st + 4 * ah);
            s.a[1] = ld16(L.qweight + (size_t)arow1 * L.stride + 8 * st + 4 * ah);
            const int g = st >> 1;
            s.sz[0] = (uint32_t)__half_as_ushort(L.scales[(size_t)arow0 * L.gs + g]) |
                      ((uint32_t)__half_as_ushort(L.zeros[(size_t)arow0 * L.gs + g]) << 16);
            s.sz[1] = (uint32_t)__half_as_ushort(L.scales[(size_t)arow1 * L.gs + g]) |
                      ((uint32_t)__half_as_ushort(L.zeros[(size_t)arow1 * L.gs + g]) << 16);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = tid + 256 * u, r = idx >> 3, c = idx & 7;
                const int col = BK * st + 8 * c;
                s.b[u] = (m0 + r < M && col < L.kq) ? ld16(X + (size_t)(m0 + r) * ldx + col) : zero4;
            }
        } else {
            const int c0 = BK * (st - nq_st);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = tid + 256 * u, r = idx >> 3, c = idx & 7;
                const int col = c0 + 8 * c;
                const int orow = min(oc0 + r, L.oc - 1);
                s.a[u] = (col < L.k) ? ld16(L.weak + (size_t)orow * L.k + col) : zero4;
                s.b[u] = (m0 + r < M && col < L.k) ? ld16(X + (size_t)(m0 + r) * ldx + L.kq + col) : zero4;
            }
        }
    };
    auto store_stage = [&](const FwdStage& s, int st, unsigned char* sA, unsigned char* sB) {
        if (st < nq_st) {
#pragma unroll
            for (int rr = 0; rr < 2; ++rr) {
                const _Float16 sc = bits_h2(s.sz[rr])[0], zp = bits_h2(s.sz[rr])[1];
                const h2 s2 = h2{sc, sc}, z2 = h2{zp, zp};
                const int r = ar + 128 * rr;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    *reinterpret_cast<u4*>(sA + tile_off(r, 4 * ah + i)) = dequant_word(s.a[rr][i], z2, s2, cst);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = tid + 256 * u, r = idx >> 3, c = idx & 7;
                *reinterpret_cast<u4*>(sB + tile_off(r, c)) = permute_x(s.b[u]);
            }
        } else {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = tid + 256 * u, r = idx >> 3, c = idx & 7;
                *reinterpret_cast<u4*>(sA + tile_off(r, c)) = s.a[u];
                *reinterpret_cast<u4*>(sB + tile_off(r, c)) = s.b[u];
            }
        }
    };

    f16v acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    FwdStage stg;
    load_stage(stg, 0);
    store_stage(stg, 0, lds, lds + 2 * TILE_BYTES);
    __syncthreads();

    const int fr = lane & 31, fk = lane >> 5;   // fragment row within a 32-row MFMA tile, k half
    for (int st = 0; st < nst; ++st) {
        const int cur = st & 1;
        const unsigned char* sA = lds + cur * TILE_BYTES;
        const unsigned char* sB = lds + 2 * TILE_BYTES + cur * TILE_BYTES;
        if (st + 1 < nst) load_stage(stg, st + 1);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            h8 a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = *reinterpret_cast<const h8*>(sA + tile_off(wm * 128 + i * 32 + fr, 2 * ks + fk));
                b[i] = *reinterpret_cast<const h8*>(sB + tile_off(wn * 128 + i * 32 + fr, 2 * ks + fk));
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (st + 1 < nst)
            store_stage(stg, st + 1, lds + (cur ^ 1) * TILE_BYTES, lds + 2 * TILE_BYTES + (cur ^ 1) * TILE_BYTES);
        __syncthreads();
    }

    // ---- epilogue: accumulator element 4*g + r of a lane is row 8*g + 4*(lane/32) + r, column lane%32
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int m = m0 + wn * 128 + j * 32 + fr;
        if (m >= M) continue;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int oc = oc0 + wm * 128 + i * 32 + 8 * g + 4 * fk;
                if (oc < L.oc) {   // OC is a multiple of 4 on this path
                    h2 lo = h2{(_Float16)acc[i][j][4 * g + 0], (_Float16)acc[i][j][4 * g + 1]};
                    h2 hi = h2{(_Float16)acc[i][j][4 * g + 2], (_Float16)acc[i][j][4 * g + 3]};
                    *reinterpret_cast<u2*>(Y + (size_t)m * ldy + oc) = u2{h2_bits(lo), h2_bits(hi)};
                }
            }
        }
    }
}

}  // namespace

bool gemm_fwd_supported(const Layer& L, int64_t M) {
    return M >= 1 && L.bits == 4 && L.g == 128 && (L.kq % 8) == 0 && (L.k % 8) == 0 && (L.oc % 8) == 0;
}

hipError_t gemm_fwd(const Layer& L, const __half* X, int64_t M, int64_t ldx, __half* Y, int64_t ldy, hipStream_t s) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)gemm_fwd_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_oc = ceil_div(L.oc, BT), tiles_m = ceil_div(M, BT);
    gemm_fwd_kernel<<<tiles_oc * tiles_m, 256, GEMM_LDS, s>>>(L, X, (int)M, ldx, Y, ldy, tiles_oc);
    return hipGetLastError();
}

bool gemm_dx_supported(const Layer&, int64_t) { return false; }
hipError_t gemm_dx(const Layer&, const __half*, int64_t, int64_t, __half*, int64_t, hipStream_t) { return hipErrorNotSupported; }
bool weak_grad_mfma_supported(int, int, int64_t) { return false; }
size_t weak_grad_mfma_workspace(int, int, int64_t) { return 0; }
hipError_t weak_grad_mfma(int, int, const __half*, int64_t, int64_t, const __half*, int64_t, void*, int, int, void*, hipStream_t) {
    return hipErrorNotSupported;
}

}  // namespace qeft
