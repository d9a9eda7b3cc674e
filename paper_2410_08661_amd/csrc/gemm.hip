// Prefill / fine-tune path (paper Sec. 3.3): the large-M products of the fused layer as tiled
// fp16 MFMA GEMMs with fp32 accumulation (tiling and LDS layout: gemm_common.h).
//
//   forward    Y [M][OC]  = X  . W^T            contraction over IC (quantized part, then weak block)
//   backward   dX[M][IC]  = dY . W              contraction over OC, through the full mixed weight
//   weak grad  dW[OC][k]  = dY^T . X[:, weak]   contraction over the M tokens (Eq. 5, weak block only)
//
// The next stage's global loads are issued before the current stage's MFMAs and converted on
// their way into LDS afterwards: the 4-bit codes are dequantized in registers, so the MFMA loop
// only ever sees plain fp16 tiles.
//
// Dequantization: codes become the exact fp16 numbers 1024 + q by or-ing exponent bits onto
// the masked nibbles (two codes per instruction), then ((1024+q) - 1024 - z) * s in packed fp16.
// Forward: a thread converts whole words of one weight row; the nibbles of a word come out in
// the order (0,4)(1,5)(2,6)(3,7) and the activations of quantized stages are permuted to match.
// Backward: the contraction runs across weight rows, so a thread takes the same word column of
// 8 consecutive rows and pairs the rows with a byte permute before the conversion; the result is
// already transposed, in natural order.
#include <type_traits>

#include "gemm_common.h"

namespace qeft {
namespace {

using namespace gemm;

// ======================================================================================= forward
struct FwdStage {
    u4 qa[2];        // quantized stage: 4 code words of rows r and r+128
    uint32_t sz[2];  // their (scale, zero-point)
    RowLoader wk;    // weak stage: fp16 weights
    RowLoader x;     // activations
};

__global__ __launch_bounds__(256) void gemm_fwd_kernel(Layer L, const __half* __restrict__ X, int M, int64_t ldx,
                                                       __half* __restrict__ Y, int64_t ldy, int tiles_oc) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int tile = xcd_tile(tiles_oc * ((M + BT - 1) / BT));
    if (tile < 0) return;
    const int t_oc = tile % tiles_oc, t_m = tile / tiles_oc;
    const int oc0 = t_oc * BT, m0 = t_m * BT;
    const int nq_st = (L.kq + BK - 1) / BK, nw_st = (L.k + BK - 1) / BK, nst = nq_st + nw_st;
    const Consts cst = make_consts();

    const int ar = tid >> 1, ah = tid & 1;  // quantized A: rows ar and ar+128, half ah of the stage's 8 words
    const int arow0 = min(oc0 + ar, L.oc - 1), arow1 = min(oc0 + ar + 128, L.oc - 1);

    auto load_stage = [&](FwdStage& s, int st) {
        if (st < nq_st) {
            s.qa[0] = ld16(L.qweight + (size_t)arow0 * L.stride + 8 * st + 4 * ah);
            s.qa[1] = ld16(L.qweight + (size_t)arow1 * L.stride + 8 * st + 4 * ah);
            const int g = st >> 1;
            s.sz[0] = (uint32_t)__half_as_ushort(L.scales[(size_t)arow0 * L.gs + g]) |
                      ((uint32_t)__half_as_ushort(L.zeros[(size_t)arow0 * L.gs + g]) << 16);
            s.sz[1] = (uint32_t)__half_as_ushort(L.scales[(size_t)arow1 * L.gs + g]) |
                      ((uint32_t)__half_as_ushort(L.zeros[(size_t)arow1 * L.gs + g]) << 16);
            s.x.load(X, ldx, m0, M, BK * st, L.kq, tid, false);   // columns past Kq belong to the weak block
        } else {
            const int c0 = BK * (st - nq_st);
            s.wk.load(L.weak, L.k, oc0, L.oc, c0, L.k, tid, true);
            s.x.load(X + L.kq, ldx, m0, M, c0, L.k, tid, false);
        }
    };
    auto store_stage = [&](const FwdStage& s, int st, unsigned char* sA, unsigned char* sB) {
        if (st < nq_st) {
#pragma unroll
            for (int rr = 0; rr < 2; ++rr) {
                const _Float16 sc = bits_h2(s.sz[rr])[0], zp = bits_h2(s.sz[rr])[1];
                const h2 s2 = h2{sc, sc}, z2 = h2{zp, zp};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t w = s.qa[rr][i];
                    u4 r;
#pragma unroll
                    for (int p = 0; p < 4; ++p) r[p] = dequant_pair(((w >> (4 * p)) & cst.mask) | cst.magic, z2, s2);
                    *reinterpret_cast<u4*>(sA + tile_off(ar + 128 * rr, 4 * ah + i)) = r;
                }
            }
            s.x.store(sB, tid, true);
        } else {
            s.wk.store(sA, tid, false);
            s.x.store(sB, tid, false);
        }
    };

    f16v acc[4][4];
    zero_acc(acc);
    FwdStage stg;
    load_stage(stg, 0);
    store_stage(stg, 0, lds, lds + 2 * TILE_BYTES);
    __syncthreads();
    for (int st = 0; st < nst; ++st) {
        const int cur = st & 1;
        if (st + 1 < nst) load_stage(stg, st + 1);
        compute_stage(lds + cur * TILE_BYTES, lds + (2 + cur) * TILE_BYTES, acc, wm, wn, lane);
        if (st + 1 < nst) store_stage(stg, st + 1, lds + (cur ^ 1) * TILE_BYTES, lds + (2 + (cur ^ 1)) * TILE_BYTES);
        __syncthreads();
    }
    store_f16(acc, Y, ldy, oc0, L.oc, m0, M, wm, wn, lane);
}

// ------------------------------------------------------------------------- forward, software-pipelined
// Same tiles, for Kq a multiple of 64.  A stage's 64 MFMAs run in four blocks of 16; between
// the blocks the thread converts a quarter of the NEXT stage's raw data (already in registers)
// into the other LDS buffer and immediately re-issues the global loads of the stage after that
// into the registers just freed, so every load has a whole stage of MFMAs to land and the
// conversion hides under the matrix pipe.  Fragment reads of block ks+1 are issued before the
// MFMAs of block ks.  No load is conditional (rows are clamped, never masked), so the compiler's
// load-counter waits are exact.  The weak block's k/64 stages follow unpipelined.
__global__ __launch_bounds__(256) void gemm_fwd_pipe_kernel(Layer L, const __half* __restrict__ X, int M, int64_t ldx,
                                                            __half* __restrict__ Y, int64_t ldy, int tiles_oc) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int tile = xcd_tile(tiles_oc * ((M + BT - 1) / BT));
    if (tile < 0) return;
    const int t_oc = tile % tiles_oc, t_m = tile / tiles_oc;
    const int oc0 = t_oc * BT, m0 = t_m * BT;
    const int nq = L.kq / BK;
    const Consts cst = make_consts();

    // quantized A: rows ar and ar+128, half ah of the stage's 8 words
    const int ar = tid >> 1, ah = tid & 1;
    const int arow[2] = {min(oc0 + ar, L.oc - 1), min(oc0 + ar + 128, L.oc - 1)};
    const uint32_t* wp[2] = {L.qweight + (size_t)arow[0] * L.stride + 4 * ah, L.qweight + (size_t)arow[1] * L.stride + 4 * ah};
    const __half* sp[2] = {L.scales + (size_t)arow[0] * L.gs, L.scales + (size_t)arow[1] * L.gs};
    const __half* zp[2] = {L.zeros + (size_t)arow[0] * L.gs, L.zeros + (size_t)arow[1] * L.gs};
    // X: chunk u of this thread is tile row (tid >> 3) + 32 u, chunk column tid & 7
    const int xr = tid >> 3, xc = tid & 7;
    const __half* xp[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) xp[u] = X + (size_t)min(m0 + xr + 32 * u, M - 1) * ldx + 8 * xc;

    u4 xv[8], av[2];
    __half sraw[2], zraw[2];   // kept as loaded: combining them here would wait for the loads at once
    auto load_a = [&](int rr, int st) {
        av[rr] = ld16(wp[rr] + 8 * st);
        sraw[rr] = sp[rr][st >> 1];
        zraw[rr] = zp[rr][st >> 1];
    };
    auto load_x = [&](int u, int st) { xv[u] = ld16(xp[u] + BK * st); };
    auto conv_a = [&](int rr, unsigned char* sA) {
        const _Float16 sc = __builtin_bit_cast(_Float16, sraw[rr]), zv = __builtin_bit_cast(_Float16, zraw[rr]);
        const h2 s2 = h2{sc, sc}, z2 = h2{zv, zv};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t w = av[rr][i];
            u4 r;
#pragma unroll
            for (int p = 0; p < 4; ++p) r[p] = dequant_pair(((w >> (4 * p)) & cst.mask) | cst.magic, z2, s2);
            *reinterpret_cast<u4*>(sA + tile_off(ar + 128 * rr, 4 * ah + i)) = r;
        }
    };
    auto conv_x = [&](int u, unsigned char* sB) {
        *reinterpret_cast<u4*>(sB + tile_off(xr + 32 * u, xc)) = permute_x(xv[u]);
    };

    f16v acc[4][4];
    zero_acc(acc);
    Frags f, fn;

    if (nq > 0) {
        // prologue: stage 0 into LDS buffer 0, stage 1 into the registers
#pragma unroll
        for (int u = 0; u < 8; ++u) load_x(u, 0);
        load_a(0, 0);
        load_a(1, 0);
#pragma unroll
        for (int u = 0; u < 8; ++u) conv_x(u, lds + 2 * TILE_BYTES);
        conv_a(0, lds);
        conv_a(1, lds);
        if (nq > 1) {
#pragma unroll
            for (int u = 0; u < 8; ++u) load_x(u, 1);
            load_a(0, 1);
            load_a(1, 1);
        }
        __syncthreads();
        load_frags(f, lds, lds + 2 * TILE_BYTES, wm, wn, lane, 0);

        // one stage: registers hold stage st+1; LOAD re-fills them with stage st+2 as they are converted
        auto stage = [&](int st, auto flags) {
            constexpr bool CONVERT = (decltype(flags)::value & 1) != 0, LOAD = (decltype(flags)::value & 2) != 0;
            const int cur = st & 1;
            const unsigned char* sA = lds + cur * TILE_BYTES;
            const unsigned char* sB = lds + (2 + cur) * TILE_BYTES;
            unsigned char* nA = lds + (cur ^ 1) * TILE_BYTES;
            unsigned char* nB = lds + (2 + (cur ^ 1)) * TILE_BYTES;
            // block 0
            load_frags(fn, sA, sB, wm, wn, lane, 1);
            mfma_block(f, acc);
            if (CONVERT) {
#pragma unroll
                for (int u = 0; u < 3; ++u) {
                    conv_x(u, nB);
                    if (LOAD) load_x(u, st + 2);
                }
            }
            __builtin_amdgcn_sched_barrier(0);   // loads stay in the block that frees their registers
            // block 1
            load_frags(f, sA, sB, wm, wn, lane, 2);
            mfma_block(fn, acc);
            if (CONVERT) {
#pragma unroll
                for (int u = 3; u < 6; ++u) {
                    conv_x(u, nB);
                    if (LOAD) load_x(u, st + 2);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            // block 2
            load_frags(fn, sA, sB, wm, wn, lane, 3);
            mfma_block(f, acc);
            if (CONVERT) {
#pragma unroll
                for (int u = 6; u < 8; ++u) {
                    conv_x(u, nB);
                    if (LOAD) load_x(u, st + 2);
                }
                conv_a(0, nA);
                if (LOAD) load_a(0, st + 2);
            }
            __builtin_amdgcn_sched_barrier(0);
            // block 3
            mfma_block(fn, acc);
            if (CONVERT) {
                conv_a(1, nA);
                if (LOAD) load_a(1, st + 2);
            }
            __syncthreads();
            if (CONVERT) load_frags(f, nA, nB, wm, wn, lane, 0);
        };
        int st = 0;
        for (; st + 2 < nq; ++st) stage(st, std::integral_constant<int, 3>{});   // convert st+1, load st+2
        if (st + 1 < nq) {
            stage(st, std::integral_constant<int, 1>{});                        // convert the last stage
            ++st;
        }
        stage(st, std::integral_constant<int, 0>{});
    }

    // ---- weak block: plain fp16 stages, one at a time --------------------------------------------
    const int nw = (L.k + BK - 1) / BK;
    for (int w = 0; w < nw; ++w) {
        RowLoader la, lb;
        la.load(L.weak, L.k, oc0, L.oc, BK * w, L.k, tid, true);
        lb.load(X + L.kq, ldx, m0, M, BK * w, L.k, tid, false);
        la.store(lds, tid, false);
        lb.store(lds + 2 * TILE_BYTES, tid, false);
        __syncthreads();
        compute_stage(lds, lds + 2 * TILE_BYTES, acc, wm, wn, lane);
        __syncthreads();
    }
    store_f16(acc, Y, ldy, oc0, L.oc, m0, M, wm, wn, lane);
}

// ======================================================================================= backward dX
// A[i = ic][k = oc] = W[oc][ic], B[j = m][k = oc] = dY[m][oc].  Thread (ko = t / 32, io = t % 32)
// produces the 8 x 8 block of 8 weight rows x one word column (8 input channels).
struct DxStage {
    uint32_t qw[8];   // quantized columns: the word of each of the 8 rows
    uint32_t sz[8];   // (scale, zero-point) of each row for this column's group
    ColLoader wk;     // weak columns: 8 rows x 8 fp16
    RowLoader dy;
};

__global__ __launch_bounds__(256) void gemm_dx_kernel(Layer L, const __half* __restrict__ dY, int M, int64_t lddy,
                                                      __half* __restrict__ dX, int64_t lddx, int tiles_ic) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int tile = xcd_tile(tiles_ic * ((M + BT - 1) / BT));
    if (tile < 0) return;
    const int t_ic = tile % tiles_ic, t_m = tile / tiles_ic;
    const int ic0 = t_ic * BT, m0 = t_m * BT;
    const int nst = (L.oc + BK - 1) / BK;
    const Consts cst = make_consts();

    const int ko = tid >> 5, io = tid & 31;
    const int ic = ic0 + 8 * io;          // first of this thread's 8 input channels
    const bool quant = ic < L.kq;         // Kq is a multiple of 8: a block is all quantized or all weak
    const int wcol = ic >> 3, grp = ic >> 7;

    auto load_stage = [&](DxStage& s, int st) {
        const int k0 = BK * st;
        if (quant) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int row = min(k0 + 8 * ko + e, L.oc - 1);   // rows past OC meet zero columns of dY
                s.qw[e] = L.qweight[(size_t)row * L.stride + wcol];
                s.sz[e] = (uint32_t)__half_as_ushort(L.scales[(size_t)row * L.gs + grp]) |
                          ((uint32_t)__half_as_ushort(L.zeros[(size_t)row * L.gs + grp]) << 16);
            }
        } else {
            s.wk.load(L.weak, L.k, k0, L.oc, ic0 - L.kq, L.k, tid);
        }
        s.dy.load(dY, lddy, m0, M, k0, L.oc, tid, false);
    };
    auto store_stage = [&](const DxStage& s, unsigned char* sA, unsigned char* sB) {
        if (quant) {
            u4 out[8];
#pragma unroll
            for (int p = 0; p < 4; ++p) {   // rows 2p and 2p+1 side by side
                const h2 s2 = h2{bits_h2(s.sz[2 * p])[0], bits_h2(s.sz[2 * p + 1])[0]};
                const h2 z2 = h2{bits_h2(s.sz[2 * p])[1], bits_h2(s.sz[2 * p + 1])[1]};
#pragma unroll
                for (int b = 0; b < 4; ++b) {   // byte b of both words: codes 2b and 2b+1
                    const uint32_t sel = 0x0c000c00u | ((4u + b) << 16) | (uint32_t)b;
                    const uint32_t t = __builtin_amdgcn_perm(s.qw[2 * p + 1], s.qw[2 * p], sel);
                    out[2 * b][p] = dequant_pair((t & cst.mask) | cst.magic, z2, s2);
                    out[2 * b + 1][p] = dequant_pair(((t >> 4) & cst.mask) | cst.magic, z2, s2);
                }
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) *reinterpret_cast<u4*>(sA + tile_off(8 * io + j, ko)) = out[j];
        } else {
            s.wk.store(sA, tid);
        }
        s.dy.store(sB, tid, false);
    };

    f16v acc[4][4];
    zero_acc(acc);
    DxStage stg;
    load_stage(stg, 0);
    store_stage(stg, lds, lds + 2 * TILE_BYTES);
    __syncthreads();
    for (int st = 0; st < nst; ++st) {
        const int cur = st & 1;
        if (st + 1 < nst) load_stage(stg, st + 1);
        compute_stage(lds + cur * TILE_BYTES, lds + (2 + cur) * TILE_BYTES, acc, wm, wn, lane);
        if (st + 1 < nst) store_stage(stg, lds + (cur ^ 1) * TILE_BYTES, lds + (2 + (cur ^ 1)) * TILE_BYTES);
        __syncthreads();
    }
    store_f16(acc, dX, lddx, ic0, L.ic, m0, M, wm, wn, lane);
}

// ======================================================================================= weak gradient
// A[i = c][k = m] = Xw[m][c], B[j = oc][k = m] = dY[m][oc]: both operands are read transposed.
// The tokens are split over `splits` workgroups per OC tile; each writes an fp32 partial
// [OC][k] slab, summed in slab order by a second kernel (no atomics: deterministic).
__global__ __launch_bounds__(256) void weak_grad_kernel(int oc_total, int k, const __half* __restrict__ dY, int M,
                                                        int64_t lddy, const __half* __restrict__ Xw, int64_t ldxw,
                                                        float* __restrict__ part, int splits, int chunk) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int split = blockIdx.x % splits, t_oc = blockIdx.x / splits;
    const int oc0 = t_oc * BT;
    const int mb = split * chunk, me = min(mb + chunk, M);
    const int nst = (me - mb + BK - 1) / BK;

    f16v acc[4][4];
    zero_acc(acc);
    ColLoader la, lb;
    if (nst > 0) {
        la.load(Xw, ldxw, mb, me, 0, k, tid);
        lb.load(dY, lddy, mb, me, oc0, oc_total, tid);
        la.store(lds, tid);
        lb.store(lds + 2 * TILE_BYTES, tid);
    }
    __syncthreads();
    for (int st = 0; st < nst; ++st) {
        const int cur = st & 1;
        if (st + 1 < nst) {
            la.load(Xw, ldxw, mb + BK * (st + 1), me, 0, k, tid);
            lb.load(dY, lddy, mb + BK * (st + 1), me, oc0, oc_total, tid);
        }
        compute_stage(lds + cur * TILE_BYTES, lds + (2 + cur) * TILE_BYTES, acc, wm, wn, lane);
        if (st + 1 < nst) {
            la.store(lds + (cur ^ 1) * TILE_BYTES, tid);
            lb.store(lds + (2 + (cur ^ 1)) * TILE_BYTES, tid);
        }
        __syncthreads();
    }
    store_f32(acc, part + (size_t)split * oc_total * k, k, 0, k, oc0, oc_total, wm, wn, lane);
}

__global__ __launch_bounds__(256) void weak_grad_reduce_kernel(const float* __restrict__ part, int splits, int64_t n,
                                                               void* dW, int out_f32, int accumulate) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    float s = 0.f;
    for (int p = 0; p < splits; ++p) s += part[(size_t)p * n + i];
    if (out_f32) {
        float* o = (float*)dW + i;
        *o = accumulate ? *o + s : s;
    } else {
        __half* o = (__half*)dW + i;
        *o = __float2half_rn(accumulate ? __half2float(*o) + s : s);
    }
}

hipError_t raise_lds_limit(const void* fn, bool& done) {
    if (done) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_LDS);
    if (e == hipSuccess) done = true;
    return e;
}

// tokens per split: whole stages, enough workgroups to cover the CUs
void weak_grad_split(int oc, int64_t M, int& splits, int& chunk) {
    const int oc_tiles = ceil_div(oc, BT);
    const int stages = ceil_div(M, BK);
    int want = ceil_div(256, oc_tiles);
    if (want > stages) want = stages;
    if (want < 1) want = 1;
    chunk = ceil_div(stages, want) * BK;
    splits = ceil_div(M, chunk);
}

}  // namespace

bool gemm_fwd_supported(const Layer& L, int64_t M) {
    return M >= 1 && L.bits == 4 && L.g == 128 && (L.kq % 8) == 0 && (L.k % 8) == 0 && (L.oc % 8) == 0;
}

hipError_t gemm_fwd(const Layer& L, const __half* X, int64_t M, int64_t ldx, __half* Y, int64_t ldy, hipStream_t s) {
    static bool attr = false;
    hipError_t e = raise_lds_limit((const void*)gemm_fwd_kernel, attr);
    if (e != hipSuccess) return e;
    const int tiles_oc = ceil_div(L.oc, BT), tiles_m = ceil_div(M, BT);
    if (L.kq > 0 && L.kq % BK == 0) {   // whole quantized stages: the software-pipelined kernel
        static bool attr2 = false;
        e = raise_lds_limit((const void*)gemm_fwd_pipe_kernel, attr2);
        if (e != hipSuccess) return e;
        gemm_fwd_pipe_kernel<<<xcd_grid(tiles_oc * tiles_m), 256, GEMM_LDS, s>>>(L, X, (int)M, ldx, Y, ldy, tiles_oc);
    } else {
        gemm_fwd_kernel<<<xcd_grid(tiles_oc * tiles_m), 256, GEMM_LDS, s>>>(L, X, (int)M, ldx, Y, ldy, tiles_oc);
    }
    return hipGetLastError();
}

bool gemm_dx_supported(const Layer& L, int64_t M) {
    return M > 16 && L.bits == 4 && L.g == 128 && (L.kq % 8) == 0 && (L.k % 8) == 0 && (L.oc % 8) == 0 &&
           (L.ic % 8) == 0;
}

hipError_t gemm_dx(const Layer& L, const __half* dY, int64_t M, int64_t lddy, __half* dX, int64_t lddx, hipStream_t s) {
    static bool attr = false;
    hipError_t e = raise_lds_limit((const void*)gemm_dx_kernel, attr);
    if (e != hipSuccess) return e;
    const int tiles_ic = ceil_div(L.ic, BT), tiles_m = ceil_div(M, BT);
    gemm_dx_kernel<<<xcd_grid(tiles_ic * tiles_m), 256, GEMM_LDS, s>>>(L, dY, (int)M, lddy, dX, lddx, tiles_ic);
    return hipGetLastError();
}

bool weak_grad_mfma_supported(int oc, int k, int64_t M) {
    return M >= 64 && k >= 8 && k <= BT && (k % 8) == 0 && (oc % 8) == 0;
}

size_t weak_grad_mfma_workspace(int oc, int k, int64_t M) {
    int splits, chunk;
    weak_grad_split(oc, M, splits, chunk);
    return (size_t)splits * oc * k * sizeof(float);
}

hipError_t weak_grad_mfma(int oc, int k, const __half* dY, int64_t M, int64_t lddy, const __half* Xw, int64_t ldxw,
                          void* dW, int out_f32, int accumulate, void* ws, hipStream_t s) {
    static bool attr = false;
    hipError_t e = raise_lds_limit((const void*)weak_grad_kernel, attr);
    if (e != hipSuccess) return e;
    int splits, chunk;
    weak_grad_split(oc, M, splits, chunk);
    weak_grad_kernel<<<ceil_div(oc, BT) * splits, 256, GEMM_LDS, s>>>(oc, k, dY, (int)M, lddy, Xw, ldxw, (float*)ws,
                                                                     splits, chunk);
    const int64_t n = (int64_t)oc * k;
    weak_grad_reduce_kernel<<<ceil_div(n, 256), 256, 0, s>>>((const float*)ws, splits, n, dW, out_f32, accumulate);
    return hipGetLastError();
}

}  // namespace qeft
