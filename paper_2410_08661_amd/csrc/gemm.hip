// Prefill / fine-tune path (paper Sec. 3.3): the large-M products of the fused layer as tiled
// fp16 MFMA GEMMs with fp32 accumulation (tiling and LDS layout: gemm_common.h).
//
//   forward    Y [M][OC]  = X  . W^T            contraction over IC (quantized part, then weak block)
//   backward   dX[M][IC]  = dY . W              contraction over OC, through the full mixed weight
//   weak grad  dW[OC][k]  = dY^T . X[:, weak]   contraction over the M tokens (Eq. 5, weak block only)
//
// Two families of kernels live here.
//   * gemm_fwd_rega_kernel / gemm_dx_rega_kernel: the 4-bit codes are dequantized straight into the
//     MFMA operand registers of the wave that multiplies them; LDS carries only the fp16 activation
//     tile (and, for dX, the raw codes transposed at 16-bit granularity).  Waves are stacked
//     along the weight rows (64 rows x 256 tokens each) so that every code is converted once;
//     software-pipelined in steps of one MFMA with static LDS / global addressing.  The forward
//     kernel can also split the K range over workgroups (few output tiles: fp16 partial tiles in a
//     workspace, summed by splitk_reduce_kernel).  Described at each kernel.
//   * gemm_fwd_kernel / gemm_dx_kernel: producer threads dequantize into an fp16 weight tile in
//     LDS.  Simpler, LDS-bound, kept for the shapes the register kernels do not take.
//
// Dequantization: codes become exact fp16 numbers by or-ing exponent bits onto masked nibbles
// (two codes per instruction): 1024 + q for a nibble at bits 0..3 of a half, 64 + q for one at
// bits 4..7 (mantissa bit 4 then weighs 1); then ((h - base) - z) * s in packed fp16: the first
// subtraction is exact, the second rounds once (exact for integer zero-points), the product once.
// The nibbles of a word come out in the order (0,4)(1,5)(2,6)(3,7); in the forward kernels the
// activations of quantized stages are permuted to match.
#include <cstdlib>
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
    int t_oc, t_m;
    tile_coords(tile, tiles_oc, (M + BT - 1) / BT, t_oc, t_m);
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

// ------------------------------------------------------------------------- forward, weights in registers
// One packed word is 8 consecutive columns of one output channel - exactly the 8 k-values one
// lane feeds into a 32x32x16 MFMA as its A operand.  So the quantized weights never touch LDS:
// lane (fr, fk) of a wave fetches, for each of its 32-row blocks, the 16 bytes holding words
// 4 fk .. 4 fk + 3 of its row for the stage, and dequantizes word ks straight into the A fragment
// of k-block ks (the k-blocks of a stage are numbered so that this works: block ks covers the
// columns of words ks and 4 + ks; the X fragments are read from LDS chunk 4 fk + ks to match).
// LDS holds only the activations (two 32 KB buffers).
//  * 4 waves stacked along the output channels, each 64 channels x 256 tokens (2 x 8 MFMA tiles):
//    every word is converted by exactly one wave, and each wave reads all eight X fragments of a
//    k-block - per MFMA the same LDS traffic as a kernel that reads both operands from LDS.
//    Conversion is what limits the kernel: measured on gfx950, a wave hides about four vector
//    instructions behind each 32x32x16 MFMA and pays in full for any more.
//  * a stage is 64 steps of one MFMA; a scheduling barrier after every step pins its share of
//    the other work: even steps read one X fragment of the next k-block and (first half of the
//    stage) permute and store half an X chunk of the next stage; odd steps convert one pair of
//    codes of the next k-block.
//  * one workgroup barrier per stage, after step 47; the last k-block reads the next stage's
//    first X fragments behind it.
//  * scales / zero-points: 8 bytes (four groups) per row and array every 8 stages, latched into a
//    packed register per row when the group changes.
struct RegConsts {
    uint32_t m0, m1, g0, g1;
};
__device__ __forceinline__ RegConsts make_reg_consts() {
    RegConsts c{0x000f000fu, 0x00f000f0u, 0x64006400u, 0x54005400u};
    asm volatile("" : "+v"(c.m0), "+v"(c.m1), "+v"(c.g0), "+v"(c.g1));
    return c;
}
// Pair P of a word (P = 0..3 -> codes (c0,c4) (c1,c5) (c2,c6) (c3,c7)); w8 = w >> 8.  Codes at bits
// 0..3 of a half become 1024 + q, codes at bits 4..7 become 64 + q (exponent chosen so that
// mantissa bit 4 weighs 1); (h - base) is exact, then - z and * s as everywhere else.
template <int P>
__device__ __forceinline__ uint32_t dequant_pair_of(uint32_t w, uint32_t w8, h2 z2, h2 s2, const RegConsts& c) {
    const h2 b0 = h2{(_Float16)1024.f, (_Float16)1024.f}, b1 = h2{(_Float16)64.f, (_Float16)64.f};
    const uint32_t src = P < 2 ? w : w8;
    const uint32_t h = (P & 1) ? ((src & c.m1) | c.g1) : ((src & c.m0) | c.g0);
    return h2_bits(((bits_h2(h) - ((P & 1) ? b1 : b0)) - z2) * s2);
}
__device__ __forceinline__ h8 dequant_word(uint32_t w, uint32_t zs, const RegConsts& c) {
    const h2 v = bits_h2(zs);
    const h2 z2 = h2{v.x, v.x}, s2 = h2{v.y, v.y};
    const uint32_t w8 = w >> 8;
    const u4 r = u4{dequant_pair_of<0>(w, w8, z2, s2, c), dequant_pair_of<1>(w, w8, z2, s2, c),
                    dequant_pair_of<2>(w, w8, z2, s2, c), dequant_pair_of<3>(w, w8, z2, s2, c)};
    return __builtin_bit_cast(h8, r);
}

constexpr int REGA_LDS = 4 * TILE_BYTES;   // X0 X1 and one tile for the weak block's weights; 32 KB per wave in the epilogue

// fp16 epilogue of a 64 (i) x 256 (j) wave tile through 32 KB of LDS of the wave's own: rows j of
// 128 bytes, 16-byte chunks XOR-swizzled with j, then 16-byte global stores (128 contiguous bytes
// per row).  QUADS = false: accumulator tile t_i row 8 g + 4 fk + e is i = 32 t_i + row; QUADS =
// true (the input-gradient kernel's quantized halves): it is i = 4 (row % 16) + t_i + 2 (row / 16).
// i0 and ni multiples of 8, out rows 16-byte aligned.  No barrier: one wave, in-order LDS.
template <bool QUADS>
__device__ __forceinline__ void store_f16_lds_64x256(const f16v (&acc)[2][8], unsigned char* stage, __half* out, int64_t ld,
                                                     int i0, int ni, int j0, int nj, int lane) {
    const int fr = lane & 31, fk = lane >> 5;
    auto pack = [](float a, float b) { return h2_bits(h2{(_Float16)a, (_Float16)b}); };
#pragma unroll
    for (int tj = 0; tj < 8; ++tj) {
        unsigned char* row = stage + (tj * 32 + fr) * 128;
        const int sw = fr & 7;
        if (!QUADS) {
#pragma unroll
            for (int ti = 0; ti < 2; ++ti)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    *reinterpret_cast<u2*>(row + (((4 * ti + g) ^ sw) << 4) + 8 * fk) =
                        u2{pack(acc[ti][tj][4 * g + 0], acc[ti][tj][4 * g + 1]), pack(acc[ti][tj][4 * g + 2], acc[ti][tj][4 * g + 3])};
        } else {
            // channels 4 c .. 4 c + 3, c = 8 g0 + 4 fk + e: (t_i, g) = (0, g0) (1, g0) (0, g0 + 2) (1, g0 + 2)
#pragma unroll
            for (int g0 = 0; g0 < 2; ++g0)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    *reinterpret_cast<u2*>(row + (((4 * g0 + 2 * fk + (e >> 1)) ^ sw) << 4) + 8 * (e & 1)) =
                        u2{pack(acc[0][tj][4 * g0 + e], acc[1][tj][4 * g0 + e]), pack(acc[0][tj][4 * (g0 + 2) + e], acc[1][tj][4 * (g0 + 2) + e])};
        }
    }
    const int c = lane & 7, r8 = lane >> 3;
    const int i = i0 + 8 * c;
#pragma unroll 8
    for (int it = 0; it < 32; ++it) {
        const int r = 8 * it + r8;
        const u4 v = *reinterpret_cast<const u4*>(stage + r * 128 + ((c ^ (r & 7)) << 4));
        if (j0 + r < nj && i < ni) *reinterpret_cast<u4*>(out + (size_t)(j0 + r) * ld + i) = v;
    }
}

// K split (splits > 1): a workgroup (tile, sp) of a split tile multiplies the quantized stages [sp * sps, (sp + 1) * sps)
// only - the last split also the weak block - and stores its partial tile as fp16 into its slot of `part` (BT rows of
// BT halves); splitk_reduce_kernel adds the partials.  Either every tile is split (launches with too few tiles to occupy
// the CUs) or only those of the last, partly filled round (split_tile).  sps is a multiple of 8 stages, so every split
// starts on a boundary of the four-group parameter fetches.
__global__ __launch_bounds__(256) void gemm_fwd_rega_kernel(Layer L, const __half* __restrict__ X, int M, int64_t ldx,
                                                            __half* __restrict__ Y, int64_t ldy, int tiles_oc, int wide_stores,
                                                            int splits, int sps, int tail_first, __half* __restrict__ part) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tiles_all = tiles_oc * ((M + BT - 1) / BT);
    int tile, sp, slot;
    if (!split_tile(tiles_all, tail_first, splits, tile, sp, slot)) return;
    int t_oc, t_m;
    tile_coords(tile, tiles_oc, (M + BT - 1) / BT, t_oc, t_m);
    const int oc0 = t_oc * BT, m0 = t_m * BT;
    const bool is_split = slot >= 0;
    const bool last_split = !is_split || sp == splits - 1;
    const int s_first = sp * sps;                                      // first stage of this workgroup
    // a layer without quantized columns (the fp16 copy of a 3-bit layer) is split along its weak stages instead:
    // a split is then the layer whose weak block starts 64 s_first columns further on
    const bool weak_split = is_split && L.kq == 0;
    const int nq = weak_split ? 0 : (is_split ? min(sps, L.kq / BK - s_first) : L.kq / BK);
    // weak stages: whole 64-column stages take the direct path below (A fragments straight from the fp16
    // block), a ragged block the LDS-staged stages at the end
    const int nwf = weak_split ? min(sps, L.k / BK - s_first) : ((L.k % BK == 0 && last_split) ? L.k / BK : 0);
    const int ns = nq + nwf;
    if (is_split) {
        // the epilogue addresses Y[m][oc] with absolute indices: point it at the slot's (m0, oc0)
        Y = part + (size_t)slot * (BT * BT) - ((size_t)m0 * BT + oc0);
        ldy = BT;
        wide_stores = 1;
    }
    const RegConsts cst = make_reg_consts();
    using lds_u4 = __attribute__((address_space(3))) u4;
    using lds_h8 = __attribute__((address_space(3))) h8;
    using gptr = const __attribute__((address_space(1))) char*;
    using g_u4 = const __attribute__((address_space(1))) u4;
    using g_u2 = const __attribute__((address_space(1))) u2;
    const int fr = lane & 31, fk = lane >> 5;

    // global addresses: wave-uniform 64-bit base (scalar registers) + 32-bit lane offset
    // (a stage is 32 bytes of codes per row, half a group = one byte of each parameter array per row, 128 bytes of X per token)
    const char* wt = reinterpret_cast<const char*>(L.qweight + (size_t)oc0 * L.stride) + 32 * s_first;
    const char* st_ = reinterpret_cast<const char*>(L.scales + (size_t)oc0 * L.gs) + s_first;
    const char* zt = reinterpret_cast<const char*>(L.zeros + (size_t)oc0 * L.gs) + s_first;
    const char* xt = reinterpret_cast<const char*>(X + (size_t)m0 * ldx) + 2 * BK * s_first;
    const char* wk = reinterpret_cast<const char*>(L.weak + (size_t)oc0 * L.k) + (weak_split ? 2 * BK * s_first : 0);
    uint32_t aoff[2], szoff[2], xoff[8];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const uint32_t row = (uint32_t)min(wave * 64 + 32 * i + fr, L.oc - 1 - oc0);
        aoff[i] = (row * (uint32_t)L.stride + 4u * fk) * 4u;
        szoff[i] = row * (uint32_t)L.gs * 2u;
    }
    const int xr = tid >> 3, xc = tid & 7;   // X chunk u of this thread: tile row xr + 32 u, chunk column xc
#pragma unroll
    for (int u = 0; u < 8; ++u) xoff[u] = ((uint32_t)min(xr + 32 * u, M - 1 - m0) * (uint32_t)ldx + 8u * xc) * 2u;
    auto sbase = [](const char* p) {
        asm volatile("" : "+s"(p));
        return (gptr)p;
    };

    // LDS addresses: base register + compile-time offset.  Rows 64 apart share the swizzle, rows
    // 32 apart differ in bit 2 of it, so chunk writes use two bases and fragment reads one base
    // per XOR constant.
    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char*)lds;
    uint32_t xw[2] = {lds0 + (uint32_t)tile_off(xr, xc), lds0 + (uint32_t)tile_off(xr + 32, xc)};
    uint32_t fb[8];
    {
        const uint32_t base = (uint32_t)((4 * fk) ^ (fr & 7) ^ (fr >> 3));
#pragma unroll
        for (int x = 0; x < 8; ++x) fb[x] = lds0 + (uint32_t)fr * 128u + ((base ^ (uint32_t)x) << 4);
    }

    u4 araw[2][2];      // codes: set = stage parity, row block i; word ks of the stage in component ks
    u4 xv[8];           // X of the stage after the current one
    u2 szs[2], szz[2];  // scales / zero-points of four consecutive groups, per row block
    uint32_t lsz[2];    // latched group: zero-point in the low half, scale in the high half
    u4 afr[2][2];       // A fragments as packed halfs, written one pair at a time
    h8 bfr[2][8];
    uint32_t cq[8];     // the conversion pipeline: one register per pair of the k-block being converted
    uint32_t w8[2];     // word >> 8 per row block
    u4 px;              // the X chunk being permuted
    auto load_a = [&](int set, int i, int st) { araw[set][i] = *reinterpret_cast<g_u4*>(sbase(wt + 32 * st) + aoff[i]); };
    auto load_x = [&](int u, int st) { xv[u] = *reinterpret_cast<g_u4*>(sbase(xt + 2 * BK * st) + xoff[u]); };
    auto load_sz = [&](int g4) {   // groups g4 .. g4 + 3 (g4 a multiple of 4; the arrays are padded to a multiple of 8 groups)
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            szs[i] = *reinterpret_cast<g_u2*>(sbase(st_ + 2 * g4) + szoff[i]);
            szz[i] = *reinterpret_cast<g_u2*>(sbase(zt + 2 * g4) + szoff[i]);
        }
    };
    auto latch = [&](int g) {
        const int sh = 16 * (g & 3);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint64_t s64 = ((uint64_t)szs[i].y << 32) | szs[i].x, z64 = ((uint64_t)szz[i].y << 32) | szz[i].x;
            lsz[i] = ((uint32_t)(z64 >> sh) & 0xffffu) | ((uint32_t)(s64 >> sh) << 16);
        }
    };
    auto put_x = [&](int u, int buf) {
        *reinterpret_cast<lds_u4*>(xw[u & 1] + (uint32_t)((u >> 1) * 8192 + buf * TILE_BYTES)) = permute_x(xv[u]);
    };
    auto read_b = [&](int set, int j, int buf, int kn) {
        bfr[set][j] = *reinterpret_cast<const lds_h8*>(fb[kn ^ (4 * (j & 1))] + (uint32_t)(j * 4096 + buf * TILE_BYTES));
    };

    f16v acc[2][8];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // weak block operands: chunk u of this thread is tile row xr + 32 u, 16-byte column xc of the stage
    // (branch-free fetches: columns past k read the row's last 8 and are zeroed when stored)
    const int nw = (nwf || !last_split) ? 0 : (L.k + BK - 1) / BK;
    const u4 zero4 = u4{0u, 0u, 0u, 0u};
    u4 wa[8], wb[8];
    auto load_weak = [&](int w) {
        const int col = min(BK * w + 8 * xc, L.k - 8);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int r = xr + 32 * u;
            wa[u] = ld16(L.weak + (size_t)min(oc0 + r, L.oc - 1) * L.k + col);
            wb[u] = ld16(X + (size_t)min(m0 + r, M - 1) * ldx + L.kq + col);
        }
    };

    if (nq > 0) {
        const int s1 = min(1, nq - 1), s1x = min(1, ns - 1);
#pragma unroll
        for (int u = 0; u < 8; ++u) load_x(u, 0);
#pragma unroll
        for (int i = 0; i < 2; ++i) load_a(0, i, 0);
        load_sz(0);
#pragma unroll
        for (int i = 0; i < 2; ++i) load_a(1, i, s1);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            put_x(u, 0);
            load_x(u, s1x);
        }
        latch(0);
#pragma unroll
        for (int i = 0; i < 2; ++i) afr[0][i] = __builtin_bit_cast(u4, dequant_word(araw[0][i].x, lsz[i], cst));
        // the pipeline finishes "the previous k-block's last pair" in its first two steps: hand it
        // that pair of the first k-block in the state it expects (masked and rebased)
        cq[7] = h2_bits(bits_h2(((araw[0][1].x >> 8) & cst.m1) | cst.g1) - h2{(_Float16)64.f, (_Float16)64.f});
#pragma unroll
        for (int e = 0; e < 7; ++e) cq[e] = 0u;
        w8[0] = w8[1] = 0u;
        px = u4{0u, 0u, 0u, 0u};
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; ++j) read_b(0, j, 0, 0);

        // stage st: X in buffer CUR, codes in set CUR
        auto stage = [&](int st, auto cur_c) {
            constexpr int CUR = decltype(cur_c)::value, NXT = CUR ^ 1;
            const int sl = min(st + 2, nq - 1), slx = min(st + 2, ns - 1);   // the activations run on into the weak stages
            // keep "base + constant" from being hoisted out of the loop into a register per constant:
            // inside the stage it folds into the instruction's offset field
            asm volatile("" : "+v"(fb[0]), "+v"(fb[1]), "+v"(fb[2]), "+v"(fb[3]), "+v"(fb[4]), "+v"(fb[5]), "+v"(fb[6]), "+v"(fb[7]));
            asm volatile("" : "+v"(xw[0]), "+v"(xw[1]), "+v"(aoff[0]), "+v"(aoff[1]));
            asm volatile("" : "+v"(xoff[0]), "+v"(xoff[1]), "+v"(xoff[2]), "+v"(xoff[3]), "+v"(xoff[4]), "+v"(xoff[5]), "+v"(xoff[6]), "+v"(xoff[7]));
            auto step = [&](auto t_c) {
                constexpr int T = decltype(t_c)::value, ks = T >> 4, t = T & 15, i = t >> 3, j = t & 7, kn = (ks + 1) & 3;
                constexpr int SRC = ks < 3 ? CUR : NXT;   // where the next k-block comes from
                if (T == 50 && CUR == 1) {
                    // the pairs converted from here on belong to the next stage, which opens a new group:
                    // latch it, and when it was the last of the four held in registers fetch the
                    // following four (needed two stages from now)
                    const int g = min(st + 1, nq - 1) >> 1;
                    latch(g);
                    if ((g & 3) == 3 && 2 * (g + 1) < nq) load_sz(g + 1);
                }
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, afr[ks & 1][i]), bfr[ks & 1][j], acc[i][j], 0, 0, 0);
                // Conversion of the next k-block's two words, software-pipelined so that no step holds
                // two dependent instructions: pair a = t / 2 is masked at step 2a, rebased at 2a + 1,
                // has its zero-point subtracted at 2a + 2 and is scaled at 2a + 3 (the last pair
                // finishes in the first two steps of the following k-block, before its row block is used).
                constexpr int a = t >> 1, ap = (a + 7) & 7;   // this step's young pair, and the one two steps older
                constexpr int aci = a >> 2, apci = ap >> 2;
                const h2 zs_old = bits_h2(lsz[apci]);
                if ((t & 1) == 0) {
                    const uint32_t w = araw[SRC][aci][kn];
                    if ((a & 3) == 1) w8[aci] = w >> 8;
                    const uint32_t src = (a & 3) < 2 ? w : w8[aci];
                    cq[a] = (a & 1) ? ((src & cst.m1) | cst.g1) : ((src & cst.m0) | cst.g0);
                    cq[ap] = h2_bits(bits_h2(cq[ap]) - h2{zs_old.x, zs_old.x});
                    read_b(kn & 1, t >> 1, SRC, kn);
                    if (T >= 4 && T <= 32 && (T & 3) == 0) {   // the chunk permuted in the two odd steps before
                        constexpr int u = (T >> 2) - 1;
                        *reinterpret_cast<lds_u4*>(xw[u & 1] + (uint32_t)((u >> 1) * 8192 + NXT * TILE_BYTES)) = px;
                    }
                } else {
                    const h2 b0 = h2{(_Float16)1024.f, (_Float16)1024.f}, b1 = h2{(_Float16)64.f, (_Float16)64.f};
                    cq[a] = h2_bits(bits_h2(cq[a]) - ((a & 1) ? b1 : b0));
                    // pair 7 of the previous conversion belongs to the k-block now being multiplied
                    afr[a == 0 ? (ks & 1) : (kn & 1)][apci][ap & 3] = h2_bits(bits_h2(cq[ap]) * h2{zs_old.y, zs_old.y});
                    if (T < 32) {   // X chunk u of the next stage: half of the permutation per odd step
                        constexpr int u = T >> 2;
                        if ((T & 2) == 0) {
                            px.x = __builtin_amdgcn_perm(xv[u].z, xv[u].x, 0x05040100u);
                            px.y = __builtin_amdgcn_perm(xv[u].z, xv[u].x, 0x07060302u);
                        } else {
                            px.z = __builtin_amdgcn_perm(xv[u].w, xv[u].y, 0x05040100u);
                            px.w = __builtin_amdgcn_perm(xv[u].w, xv[u].y, 0x07060302u);
                            load_x(u, slx);
                        }
                    }
                    if (ks == 3 && j == 7) load_a(CUR, i, sl);
                }
                if (T == 47) __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
            };
            auto steps8 = [&](auto b_c) {
                constexpr int B = decltype(b_c)::value;
                step(std::integral_constant<int, B + 0>{});
                step(std::integral_constant<int, B + 1>{});
                step(std::integral_constant<int, B + 2>{});
                step(std::integral_constant<int, B + 3>{});
                step(std::integral_constant<int, B + 4>{});
                step(std::integral_constant<int, B + 5>{});
                step(std::integral_constant<int, B + 6>{});
                step(std::integral_constant<int, B + 7>{});
            };
            steps8(std::integral_constant<int, 0>{});
            steps8(std::integral_constant<int, 8>{});
            steps8(std::integral_constant<int, 16>{});
            steps8(std::integral_constant<int, 24>{});
            steps8(std::integral_constant<int, 32>{});
            steps8(std::integral_constant<int, 40>{});
            steps8(std::integral_constant<int, 48>{});
            steps8(std::integral_constant<int, 56>{});
        };
        int st = 0;
        for (; st + 1 < nq; st += 2) {
            stage(st, std::integral_constant<int, 0>{});
            stage(st + 1, std::integral_constant<int, 1>{});
        }
        if (nq & 1) stage(st, std::integral_constant<int, 0>{});
        if (nwf == 0) __syncthreads();
    }

    // ---- weak block, whole stages: the same 64-step stage without a conversion ------------------------
    // The activation pipeline above simply runs on (the weak columns follow the quantized ones in X), so the
    // tiles keep the chunk order of the 4-bit conversion.  A lane's A fragment of k-block kn is 16 contiguous
    // bytes of its row of the fp16 block: it is fetched one stage ahead into the register of the k-block just
    // consumed and brought into the tiles' chunk order by four byte permutes while the previous k-block is
    // multiplied.  No weight passes through LDS.
    if (nwf > 0) {
        u4 wfr[2][4];      // [row block][k-block]
        uint32_t woff[2];  // (computed here: the stage loop above has no register to carry them)
#pragma unroll
        for (int i = 0; i < 2; ++i)
            woff[i] = ((uint32_t)min(wave * 64 + 32 * i + fr, L.oc - 1 - oc0) * (uint32_t)L.k + 32u * fk) * 2u;
        auto load_w = [&](int i, int kn, uint32_t off) {   // scalar base + lane offset + immediate
            wfr[i][kn] = *reinterpret_cast<g_u4*>(((gptr)wk + off) + 16 * kn);
        };
        auto order_w = [&](int i, int kn, int dst) {   // A fragment in the tiles' chunk order
            const u4 v = wfr[i][kn];
            afr[dst][i].x = __builtin_amdgcn_perm(v.z, v.x, 0x05040100u);
            afr[dst][i].y = __builtin_amdgcn_perm(v.z, v.x, 0x07060302u);
            afr[dst][i].z = __builtin_amdgcn_perm(v.w, v.y, 0x05040100u);
            afr[dst][i].w = __builtin_amdgcn_perm(v.w, v.y, 0x07060302u);
        };
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int kn = 0; kn < 4; ++kn) load_w(i, kn, woff[i]);
        if (nq == 0) {   // no stage has run yet: start the activation pipeline here
            const int s1x = min(1, ns - 1);
#pragma unroll
            for (int u = 0; u < 8; ++u) load_x(u, 0);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                put_x(u, 0);
                load_x(u, s1x);
            }
            px = u4{0u, 0u, 0u, 0u};
            __syncthreads();
#pragma unroll
            for (int j = 0; j < 8; ++j) read_b(0, j, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            order_w(i, 0, 0);
            load_w(i, 0, woff[i] + (uint32_t)(2 * BK * min(1, nwf - 1)));
        }

        // weak stage w: X in buffer CUR
        auto wstage = [&](int w, auto cur_c) {
            constexpr int CUR = decltype(cur_c)::value, NXT = CUR ^ 1;
            const int slx = min(nq + w + 2, ns - 1);
            uint32_t wo1[2], wo2[2];   // this thread's rows in the next stage and in the one after
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                wo1[i] = woff[i] + (uint32_t)(2 * BK * min(w + 1, nwf - 1));
                wo2[i] = woff[i] + (uint32_t)(2 * BK * min(w + 2, nwf - 1));
            }
            asm volatile("" : "+v"(fb[0]), "+v"(fb[1]), "+v"(fb[2]), "+v"(fb[3]), "+v"(fb[4]), "+v"(fb[5]), "+v"(fb[6]), "+v"(fb[7]));
            asm volatile("" : "+v"(xw[0]), "+v"(xw[1]), "+v"(wo1[0]), "+v"(wo1[1]), "+v"(wo2[0]), "+v"(wo2[1]));
            asm volatile("" : "+v"(xoff[0]), "+v"(xoff[1]), "+v"(xoff[2]), "+v"(xoff[3]), "+v"(xoff[4]), "+v"(xoff[5]), "+v"(xoff[6]), "+v"(xoff[7]));
            auto step = [&](auto t_c) {
                constexpr int T = decltype(t_c)::value, ks = T >> 4, t = T & 15, i = t >> 3, j = t & 7, kn = (ks + 1) & 3;
                constexpr int SRC = ks < 3 ? CUR : NXT;          // tile of the next k-block
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, afr[ks & 1][i]), bfr[ks & 1][j], acc[i][j], 0, 0, 0);
                if ((t & 1) == 0) {
                    read_b(kn & 1, t >> 1, SRC, kn);
                    if (T >= 4 && T <= 32 && (T & 3) == 0) {   // the chunk permuted in the two odd steps before
                        constexpr int u = (T >> 2) - 1;
                        *reinterpret_cast<lds_u4*>(xw[u & 1] + (uint32_t)((u >> 1) * 8192 + NXT * TILE_BYTES)) = px;
                    }
                    // the next k-block's fragments (k-block 0 of the next stage behind the last one), one row block
                    // per step; each register is then refilled with the same k-block one stage on
                    if (t == 4) order_w(0, kn, kn & 1);
                    if (t == 6) order_w(1, kn, kn & 1);
                    if (t == 10) load_w(0, kn, ks < 3 ? wo1[0] : wo2[0]);
                    if (t == 12) load_w(1, kn, ks < 3 ? wo1[1] : wo2[1]);
                } else {
                    if (T < 32) {   // X chunk u of the next stage: half of the permutation per odd step
                        constexpr int u = T >> 2;
                        if ((T & 2) == 0) {
                            px.x = __builtin_amdgcn_perm(xv[u].z, xv[u].x, 0x05040100u);
                            px.y = __builtin_amdgcn_perm(xv[u].z, xv[u].x, 0x07060302u);
                        } else {
                            px.z = __builtin_amdgcn_perm(xv[u].w, xv[u].y, 0x05040100u);
                            px.w = __builtin_amdgcn_perm(xv[u].w, xv[u].y, 0x07060302u);
                            load_x(u, slx);
                        }
                    }
                }
                if (T == 47) __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
            };
            auto steps8 = [&](auto b_c) {
                constexpr int B = decltype(b_c)::value;
                step(std::integral_constant<int, B + 0>{});
                step(std::integral_constant<int, B + 1>{});
                step(std::integral_constant<int, B + 2>{});
                step(std::integral_constant<int, B + 3>{});
                step(std::integral_constant<int, B + 4>{});
                step(std::integral_constant<int, B + 5>{});
                step(std::integral_constant<int, B + 6>{});
                step(std::integral_constant<int, B + 7>{});
            };
            steps8(std::integral_constant<int, 0>{});
            steps8(std::integral_constant<int, 8>{});
            steps8(std::integral_constant<int, 16>{});
            steps8(std::integral_constant<int, 24>{});
            steps8(std::integral_constant<int, 32>{});
            steps8(std::integral_constant<int, 40>{});
            steps8(std::integral_constant<int, 48>{});
            steps8(std::integral_constant<int, 56>{});
        };
        int w = 0;
        if (nq & 1) {   // the first weak stage sits in tile 1
            wstage(0, std::integral_constant<int, 1>{});
            w = 1;
        }
        for (; w + 1 < nwf; w += 2) {
            wstage(w, std::integral_constant<int, 0>{});
            wstage(w + 1, std::integral_constant<int, 1>{});
        }
        if (w < nwf) wstage(w, std::integral_constant<int, 0>{});
        __syncthreads();
    }
    if (nw > 0) load_weak(0);

    // ---- weak block: plain fp16 stages with both operands through LDS -------------------------------
    // Stage w sits in tiles (w & 1) [X] and 2 + (w & 1) [weights].  While its four k-blocks are
    // multiplied (fragments read one block ahead), stage w + 1 moves from the registers into the
    // other pair of tiles, a quarter per k-block, and stage w + 2 is fetched.
    auto store_weak = [&](int w, int q) {   // chunks 2 q, 2 q + 1 of this thread, of stage w
        unsigned char* sB = lds + (w & 1) * TILE_BYTES;
        unsigned char* sA = lds + (2 + (w & 1)) * TILE_BYTES;
        const bool ok = BK * w + 8 * xc < L.k;
#pragma unroll
        for (int u = 2 * q; u < 2 * q + 2; ++u) {
            *reinterpret_cast<u4*>(sA + tile_off(xr + 32 * u, xc)) = ok ? wa[u] : zero4;
            *reinterpret_cast<u4*>(sB + tile_off(xr + 32 * u, xc)) = ok ? wb[u] : zero4;
        }
    };
    if (nw > 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) store_weak(0, q);
        if (nw > 1) load_weak(1);
        __syncthreads();
    }
    for (int w = 0; w < nw; ++w) {
        const unsigned char* sB = lds + (w & 1) * TILE_BYTES;
        const unsigned char* sA = lds + (2 + (w & 1)) * TILE_BYTES;
        FragsT<2, 8> f[2];
        load_frags_t<2, 8>(f[0], sA, sB, wave * 64, 0, lane, 0);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks < 3) load_frags_t<2, 8>(f[(ks + 1) & 1], sA, sB, wave * 64, 0, lane, ks + 1);
            mfma_block_t<2, 8>(f[ks & 1], acc);
            if (w + 1 < nw) store_weak(w + 1, ks);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (w + 2 < nw) load_weak(w + 2);
        if (w + 1 < nw) __syncthreads();
    }
    if (wide_stores) __syncthreads();   // the epilogue reuses the tiles
    if (wide_stores)
        store_f16_lds_64x256<false>(acc, lds + wave * TILE_BYTES, Y, ldy, oc0 + wave * 64, L.oc, m0, M, lane);
    else
        store_f16_t<2, 8>(acc, Y, ldy, oc0 + wave * 64, L.oc, m0, M, lane);
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
                                                      __half* __restrict__ dX, int64_t lddx, int tiles_ic, int ic_start) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int tile = xcd_tile(tiles_ic * ((M + BT - 1) / BT));
    if (tile < 0) return;
    int t_ic, t_m;
    tile_coords(tile, tiles_ic, (M + BT - 1) / BT, t_ic, t_m);
    const int ic0 = ic_start + t_ic * BT, m0 = t_m * BT;
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

// ------------------------------------------------------------------------- backward dX, weights in registers
// C[i = ic][j = m] = sum_oc W[oc][ic] dY[m][oc].  The A operand of a 32x32x16 MFMA wants, per
// lane, 8 consecutive k = 8 consecutive weight ROWS of one input channel, while the stored
// matrices run along the channels.  Both kinds of weight therefore pass through LDS as "lines":
// one line holds, for the stage's 64 rows, one 16-bit column of the stored matrix, two rows to a
// 32-bit word - so 16 bytes of a line are 8 consecutive rows, paired along k.
//  * Quantized half (128 channels = 16 word columns, one group): line (W, h) is the 16-bit half h
//    of word column W, i.e. raw 4-bit codes, an eighth of the fp16 tile.  Lane (fr, fk) reads rows
//    16 ks + 8 fk .. + 7 of line (fr / 2, fr % 2): four registers whose nibble i (of both halves)
//    is channel 4 fr + i.  A fragment i is then one mask-and-or per register (no permute), and a
//    lane's four accumulators for fixed (row, column) are four consecutive channels of dX.
//    Scales and zero-points vary along k here: they are staged as fp16 vectors per row.
//  * Weak half (128 fp16 channels): a line is simply one channel; 16 bytes of it are an A fragment
//    as it stands.  Fragment i of lane fr is channel fr + 32 i.
// Everything else is the forward kernel's pipeline: 4 waves of 128 x 128, 16 slots of four MFMAs
// per stage, quantized fragments converted three slots ahead, dY staged through LDS unchanged,
// one barrier per stage after slot 11.  A tile is 256 channels = two halves, each quantized or
// weak (Kq is a multiple of 128 here); the two waves that own a half follow its kind.
// Requires OC % 64 == 0, Kq % 128 == 0 and k % 8 == 0.
constexpr int DX_LINE = 144;                      // 64 rows x 2 bytes + 16: consecutive lines 4 banks apart
constexpr int DX_HALF = 128 * DX_LINE;            // lines of one half (a quantized half uses the first 32)
constexpr int DX_LINES = 2 * DX_HALF;
constexpr int DX_SZ = 2 * 2 * 64 * 2;             // [half][zero, scale][row] fp16
constexpr int DX_LINE_BASE = 2 * TILE_BYTES;      // dY0 dY1 | lines0 lines1 | sz0 sz1
constexpr int DX_SZ_BASE = DX_LINE_BASE + 2 * DX_LINES;
constexpr int DX_LDS = DX_SZ_BASE + 2 * DX_SZ;

template <int H0, int H1>   // kinds of the tile's two halves: 0 quantized, 1 weak
__device__ __forceinline__ void dx_tile(const Layer& L, const __half* __restrict__ dY, int M, int64_t lddy,
                                        __half* __restrict__ dX, int64_t lddx, int ic0, int m0, unsigned char* lds) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = wave >> 1, lb = wave & 1;   // the tile half this wave works in, and which 64 channels of it
    const int nst = L.oc / BK;
    const RegConsts cst = make_reg_consts();
    using lds_u4 = __attribute__((address_space(3))) u4;
    using lds_u32 = __attribute__((address_space(3))) uint32_t;
    using lds_u16 = __attribute__((address_space(3))) unsigned short;
    using lds_h8 = __attribute__((address_space(3))) h8;
    using gptr = const __attribute__((address_space(1))) char*;
    using g_u4 = const __attribute__((address_space(1))) u4;
    using g_u16 = const __attribute__((address_space(1))) unsigned short;
    constexpr bool ANYQ = H0 == 0 || H1 == 0;
    constexpr int NW = 2 * (H0 + H1);   // weak items per thread: (row pair, 8 channels) blocks
    const int fr = lane & 31, fk = lane >> 5;
    auto sbase = [](const char* p) {
        asm volatile("" : "+s"(p));
        return (gptr)p;
    };

    // ---- producers: global addresses (wave-uniform 64-bit base + 32-bit lane offset) ---------------
    // dY: chunk u of this thread is tile row xr + 32 u, chunk column xc
    const int xr = tid >> 3, xc = tid & 7;
    const char* dyt = reinterpret_cast<const char*>(dY + (size_t)m0 * lddy);
    uint32_t dyoff[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) dyoff[u] = ((uint32_t)min(xr + 32 * u, M - 1 - m0) * (uint32_t)lddy + 8u * xc) * 2u;
    // codes: rows 2 rp, 2 rp + 1 of the stage, word columns 4 xc .. 4 xc + 3 of the tile, i.e. of half
    // xc / 4 (columns past the stored row are clamped; such channels are never stored)
    const int rp = tid >> 3;
    const bool code_thread = H0 == 0 && (H1 == 0 || xc < 4);
    uint32_t coff = ((uint32_t)(2 * rp) * (uint32_t)L.stride + (uint32_t)min((ic0 >> 3) + 4 * xc, L.stride - 4)) * 4u;
    const char* wt = reinterpret_cast<const char*>(L.qweight);
    const size_t wstage = (size_t)BK * L.stride * 4, wrow = (size_t)L.stride * 4;
    // scales / zero-points: thread (row = tid % 64, half = tid / 64 % 2) of waves 0 and 1
    const bool sz_wave = H0 == 0 && (H1 == 0 ? wave < 2 : wave < 1);
    uint32_t szoff = ((uint32_t)(tid & 63) * (uint32_t)L.gs + (uint32_t)min((ic0 >> 7) + ((tid >> 6) & 1), L.gs - 1)) * 2u;
    const char* st_ = reinterpret_cast<const char*>(L.scales);
    const char* zt = reinterpret_cast<const char*>(L.zeros);
    const size_t szstage = (size_t)BK * L.gs * 2;
    // weak: item n of this thread is rows 2 rp, 2 rp + 1 x channels 8 c .. 8 c + 7 of a weak half,
    // c = xc + 8 (n % 2); the halves in the order they are weak (channel blocks past k are clamped)
    uint32_t woff[NW > 0 ? NW : 1];
    const char* wkt = reinterpret_cast<const char*>(L.weak);
    const size_t wkstage = (size_t)BK * L.k * 2, wkrow = (size_t)L.k * 2;
#pragma unroll
    for (int n = 0; n < NW; ++n) {
        const int half = (H0 == 1) ? n / 2 : 1;
        const int kc = ic0 + 128 * half - L.kq + 8 * (xc + 8 * (n & 1));
        woff[n] = ((uint32_t)(2 * rp) * (uint32_t)L.k + (uint32_t)max(min(kc, L.k - 8), 0)) * 2u;
    }

    // ---- LDS addresses: base register + compile-time offset ---------------------------------------
    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char*)lds;
    uint32_t xw[2] = {lds0 + (uint32_t)tile_off(xr, xc), lds0 + (uint32_t)tile_off(xr + 32, xc)};
    uint32_t fb[4];   // dY fragments, indexed by (XOR constant) / 2
#pragma unroll
    for (int x = 0; x < 4; ++x)
        fb[x] = lds0 + (uint32_t)fr * 128u + ((((uint32_t)(fk ^ (fr & 7) ^ (fr >> 3))) ^ (2u * x)) << 4);
    // lines: the 16-byte chunk t of a line (rows 8 t .. 8 t + 7) sits at slot t ^ (line / 8 % 8), so that
    // the eight threads that write one row pair into eight different line groups spread over the banks
    const uint32_t lw = (((uint32_t)((rp >> 2) ^ xc)) << 4) + (uint32_t)(rp & 3) * 4u;   // position of row pair rp, line group xc (mod 8)
    uint32_t cwr = lds0 + DX_LINE_BASE + (uint32_t)(xc >> 2) * DX_HALF + (uint32_t)(8 * (xc & 3)) * DX_LINE + lw;
    uint32_t wwr[NW > 0 ? NW : 1];
#pragma unroll
    for (int n = 0; n < NW; ++n) {
        const int half = (H0 == 1) ? n / 2 : 1;
        wwr[n] = lds0 + DX_LINE_BASE + (uint32_t)half * DX_HALF + (uint32_t)(8 * (xc + 8 * (n & 1))) * DX_LINE + lw;
    }
    uint32_t szw = lds0 + DX_SZ_BASE + (uint32_t)((tid >> 6) & 1) * 256u + (uint32_t)(tid & 63) * 2u;

    u4 dyv[8];            // dY of the stage after the current one
    u4 cw0, cw1;          // its code words (two rows)
    unsigned short sv, zv;
    u4 ww[NW > 0 ? NW : 1][2];   // its weak blocks (two rows each)
    auto load_dy = [&](int u, int st) { dyv[u] = *reinterpret_cast<g_u4*>(sbase(dyt + 2 * BK * st) + dyoff[u]); };
    auto load_codes = [&](int st) {
        if (code_thread) {
            cw0 = *reinterpret_cast<g_u4*>(sbase(wt + st * wstage) + coff);
            cw1 = *reinterpret_cast<g_u4*>(sbase(wt + st * wstage + wrow) + coff);
        }
    };
    auto load_sz = [&](int st) {
        if (sz_wave) {
            sv = *reinterpret_cast<g_u16*>(sbase(st_ + st * szstage) + szoff);
            zv = *reinterpret_cast<g_u16*>(sbase(zt + st * szstage) + szoff);
        }
    };
    auto load_weak = [&](int n, int st) {
        ww[n][0] = *reinterpret_cast<g_u4*>(sbase(wkt + st * wkstage) + woff[n]);
        ww[n][1] = *reinterpret_cast<g_u4*>(sbase(wkt + st * wkstage + wkrow) + woff[n]);
    };
    auto put_dy = [&](int u, int buf) {
        *reinterpret_cast<lds_u4*>(xw[u & 1] + (uint32_t)((u >> 1) * 8192 + buf * TILE_BYTES)) = dyv[u];
    };
    auto put_codes = [&](int q, int buf) {   // word column 4 xc + q: low halves of both rows, high halves
        if (code_thread) {
            *reinterpret_cast<lds_u32*>(cwr + (uint32_t)((2 * q) * DX_LINE + buf * DX_LINES)) =
                __builtin_amdgcn_perm(cw1[q], cw0[q], 0x05040100u);
            *reinterpret_cast<lds_u32*>(cwr + (uint32_t)((2 * q + 1) * DX_LINE + buf * DX_LINES)) =
                __builtin_amdgcn_perm(cw1[q], cw0[q], 0x07060302u);
        }
    };
    auto put_sz = [&](int buf) {
        if (sz_wave) {
            *reinterpret_cast<lds_u16*>(szw + (uint32_t)(buf * DX_SZ)) = zv;
            *reinterpret_cast<lds_u16*>(szw + (uint32_t)(128 + buf * DX_SZ)) = sv;
        }
    };
    auto put_weak = [&](int n, int buf) {    // channel e of the block: rows 2 rp | 2 rp + 1
#pragma unroll
        for (int e = 0; e < 8; ++e)
            *reinterpret_cast<lds_u32*>(wwr[n] + (uint32_t)(e * DX_LINE + buf * DX_LINES)) =
                __builtin_amdgcn_perm(ww[n][1][e >> 1], ww[n][0][e >> 1], (e & 1) ? 0x07060302u : 0x05040100u);
    };

    f16v acc[2][8];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // ---- stage 0 into buffer 0, stage 1 into the registers ------------------------------------------
    {
        const int s1 = min(1, nst - 1);
#pragma unroll
        for (int u = 0; u < 8; ++u) load_dy(u, 0);
        if (ANYQ) {
            load_codes(0);
            load_sz(0);
        }
#pragma unroll
        for (int n = 0; n < NW; ++n) load_weak(n, 0);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            put_dy(u, 0);
            load_dy(u, s1);
        }
        if (ANYQ) {
#pragma unroll
            for (int q = 0; q < 4; ++q) put_codes(q, 0);
            load_codes(s1);
            put_sz(0);
            load_sz(s1);
        }
#pragma unroll
        for (int n = 0; n < NW; ++n) {
            put_weak(n, 0);
            load_weak(n, s1);
        }
        __syncthreads();
    }

    // this slot's share of staging stage st+1 into buffer NXT and fetching stage sl
    auto produce = [&](auto s_c, auto nxt_c, int sl) {
        constexpr int S = decltype(s_c)::value, NXT = decltype(nxt_c)::value;
        if (S < 8) {
            put_dy(S, NXT);
            load_dy(S, sl);
        }
        if (ANYQ) {
            if (S == 8) {
                put_codes(0, NXT);
                put_codes(1, NXT);
            } else if (S == 9) {
                put_codes(2, NXT);
                put_codes(3, NXT);
                load_codes(sl);
            } else if (S == 10) {
                put_sz(NXT);
                load_sz(sl);
            }
        }
        constexpr int n = S - (12 - NW);   // weak items in the last slots before the barrier
        if (NW > 0 && n >= 0 && n < NW) {
            put_weak(n, NXT);
            load_weak(n, sl);
        }
    };
    auto protect = [&]() {   // keep "base + constant" out of loop-invariant registers: it folds into the offset field
        asm volatile("" : "+v"(fb[0]), "+v"(fb[1]), "+v"(fb[2]), "+v"(fb[3]), "+v"(xw[0]), "+v"(xw[1]), "+v"(cwr), "+v"(szw), "+v"(coff), "+v"(szoff));
        asm volatile("" : "+v"(dyoff[0]), "+v"(dyoff[1]), "+v"(dyoff[2]), "+v"(dyoff[3]), "+v"(dyoff[4]), "+v"(dyoff[5]), "+v"(dyoff[6]), "+v"(dyoff[7]));
#pragma unroll
        for (int n = 0; n < NW; ++n) asm volatile("" : "+v"(woff[n]), "+v"(wwr[n]));
    };
    // ---- consumers: wave w owns 64 channels (block lb = w % 2 of half w / 2) x all 256 tokens --------
    // A stage is 64 steps of one MFMA (k-block T / 16, channel fragment T / 8 % 2, token fragment
    // T % 8) with a scheduling barrier after each: even steps read one dY fragment of the next
    // k-block, odd steps 4 S + 1 carry the producers' slot S, and the conversion of the next
    // k-block's codes is spread so that no step holds two dependent instructions.
    h8 bfr[2][8];
    u4 afr[2][2];   // A fragments of a k-block (set = block parity), as packed halfs
    auto read_b = [&](int set, int j, int buf, int kn) {
        bfr[set][j] = *reinterpret_cast<const lds_h8*>(fb[kn ^ (2 * (j & 1))] + (uint32_t)(j * 4096 + buf * TILE_BYTES));
    };
    const int icw = ic0 + 128 * half + 64 * lb;
    auto mfma_step = [&](auto t_c) {
        constexpr int T = decltype(t_c)::value, ks = T >> 4, i = (T >> 3) & 1, j = T & 7;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, afr[ks & 1][i]), bfr[ks & 1][j], acc[i][j], 0, 0, 0);
    };
    auto produce_step = [&](auto t_c, auto nxt_c, int sl) {
        constexpr int T = decltype(t_c)::value;
        if ((T & 3) == 1 && T < 48) produce(std::integral_constant<int, (T >> 2)>{}, nxt_c, sl);
    };
    auto run_stages = [&](auto&& stage) {
        int st = 0;
        for (; st + 1 < nst; st += 2) {
            stage(st, std::integral_constant<int, 0>{});
            stage(st + 1, std::integral_constant<int, 1>{});
        }
        if (nst & 1) stage(st, std::integral_constant<int, 0>{});
        __syncthreads();   // every wave is done with the staging buffers
    };
#define QEFT_STEPS8(F, B)                                                                                        \
    F(std::integral_constant<int, (B) + 0>{}); F(std::integral_constant<int, (B) + 1>{});                       \
    F(std::integral_constant<int, (B) + 2>{}); F(std::integral_constant<int, (B) + 3>{});                       \
    F(std::integral_constant<int, (B) + 4>{}); F(std::integral_constant<int, (B) + 5>{});                       \
    F(std::integral_constant<int, (B) + 6>{}); F(std::integral_constant<int, (B) + 7>{});
#define QEFT_STEPS64(F)                                                                                          \
    QEFT_STEPS8(F, 0) QEFT_STEPS8(F, 8) QEFT_STEPS8(F, 16) QEFT_STEPS8(F, 24) QEFT_STEPS8(F, 32) QEFT_STEPS8(F, 40) \
    QEFT_STEPS8(F, 48) QEFT_STEPS8(F, 56)

    // ---- a wave in a quantized half ---------------------------------------------------------------------
    // Lane fr reads line 16 lb + fr % 16 (both lanes fr and fr + 16 the same one) and takes nibble
    // t + 2 (fr / 16) of its 16-bit words for fragment t: after a per-lane shift by 0 or 8 bits,
    // fragment 0 is the nibble at bits 0..3 (as 1024 + q) and fragment 1 the one at bits 4..7 (as
    // 64 + q), the two positions that lie inside the fp16 mantissa.  Row fr of fragment t is channel
    // 4 (fr % 16) + t + 2 (fr / 16) of the wave's 64, so a lane's accumulators (0, g, e) (1, g, e)
    // (0, g + 2, e) (1, g + 2, e) are four consecutive channels.
    auto run_quant = [&]() {
        uint32_t crd[4];  // code lines, indexed by k-block
        {
            const int ln = 16 * lb + (fr & 15);
            const int cl = (ln >> 3) + 4 * half;   // the line's group in the chunk swizzle: its writer's xc
#pragma unroll
            for (int kn = 0; kn < 4; ++kn)
                crd[kn] = lds0 + DX_LINE_BASE + (uint32_t)half * DX_HALF + (uint32_t)ln * DX_LINE + ((uint32_t)((fk ^ cl) ^ (2 * kn)) << 4);
        }
        uint32_t szr = lds0 + DX_SZ_BASE + (uint32_t)half * 256u + 16u * fk;
        uint32_t nsh = 8u * (uint32_t)(fr >> 4);
        u4 cf;            // code words of the k-block being converted: register p = rows 2p | 2p+1
        u4 cfs;           // ... shifted to this lane's nibbles
        h8 zf, sf;        // zero-points and scales of its 8 rows
        uint32_t cq[8];   // the conversion pipeline, one register per pair
        auto read_codes = [&](int buf, int kn) {
            cf = *reinterpret_cast<const lds_u4*>(crd[kn] + (uint32_t)(buf * DX_LINES));
            zf = *reinterpret_cast<const lds_h8*>(szr + (uint32_t)(32 * kn + buf * DX_SZ));
            sf = *reinterpret_cast<const lds_h8*>(szr + (uint32_t)(128 + 32 * kn + buf * DX_SZ));
        };
        const h2 b0 = h2{(_Float16)1024.f, (_Float16)1024.f}, b1 = h2{(_Float16)64.f, (_Float16)64.f};
        // pair a = 4 t + p (fragment t, register p) goes through: mask, rebase, zero-point, scale
        auto cv_mask = [&](auto a_c) {
            constexpr int a = decltype(a_c)::value;
            cq[a] = (a < 4) ? ((cfs[a & 3] & cst.m0) | cst.g0) : ((cfs[a & 3] & cst.m1) | cst.g1);
        };
        auto cv_base = [&](auto a_c) {
            constexpr int a = decltype(a_c)::value;
            cq[a] = h2_bits(bits_h2(cq[a]) - (a < 4 ? b0 : b1));
        };
        auto cv_zero = [&](auto a_c) {
            constexpr int a = decltype(a_c)::value, p = a & 3;
            cq[a] = h2_bits(bits_h2(cq[a]) - h2{zf[2 * p], zf[2 * p + 1]});
        };
        auto cv_scale = [&](auto a_c, int set) {
            constexpr int a = decltype(a_c)::value, p = a & 3;
            afr[set][a >> 2][p] = h2_bits(bits_h2(cq[a]) * h2{sf[2 * p], sf[2 * p + 1]});
        };
        // pair a enters the pipeline at step 4 + a of the k-block (the lines are read at step 0, shifted
        // at step 3) and leaves it at step 7 + a <= 14
        auto convert_step = [&](auto t_c, int buf_src) {
            constexpr int T = decltype(t_c)::value, ks = T >> 4, t = T & 15, kn = (ks + 1) & 3;
            if (t == 0) read_codes(buf_src, kn);
            if (t == 3) {
#pragma unroll
                for (int p = 0; p < 4; ++p) cfs[p] = cf[p] >> nsh;
            }
            if (t >= 4 && t <= 11) cv_mask(std::integral_constant<int, (t - 4) & 7>{});
            if (t >= 5 && t <= 12) cv_base(std::integral_constant<int, (t - 5) & 7>{});
            if (t >= 6 && t <= 13) cv_zero(std::integral_constant<int, (t - 6) & 7>{});
            if (t >= 7 && t <= 14) cv_scale(std::integral_constant<int, (t - 7) & 7>{}, kn & 1);
        };
        // k-block 0 of stage 0, unpipelined
        read_codes(0, 0);
#pragma unroll
        for (int j = 0; j < 8; ++j) read_b(0, j, 0, 0);
#pragma unroll
        for (int p = 0; p < 4; ++p) cfs[p] = cf[p] >> nsh;
        QEFT_STEPS8(cv_mask, 0)
        QEFT_STEPS8(cv_base, 0)
        QEFT_STEPS8(cv_zero, 0)
        {
            auto sc0 = [&](auto a_c) { cv_scale(a_c, 0); };
            QEFT_STEPS8(sc0, 0)
        }

        auto stage = [&](int st, auto cur_c) {
            constexpr int CUR = decltype(cur_c)::value, NXT = CUR ^ 1;
            const int sl = min(st + 2, nst - 1);
            protect();
            asm volatile("" : "+v"(crd[0]), "+v"(crd[1]), "+v"(crd[2]), "+v"(crd[3]), "+v"(szr));
            auto step = [&](auto t_c) {
                constexpr int T = decltype(t_c)::value, ks = T >> 4, t = T & 15, kn = (ks + 1) & 3;
                constexpr int SRC = ks < 3 ? CUR : NXT;   // where the next k-block comes from
                mfma_step(t_c);
                if ((t & 1) == 0) read_b(kn & 1, t >> 1, SRC, kn);
                convert_step(t_c, SRC);
                produce_step(t_c, std::integral_constant<int, NXT>{}, sl);
                if (T == 47) __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
            };
            QEFT_STEPS64(step)
        };
        run_stages(stage);
        store_f16_lds_64x256<true>(acc, lds + wave * TILE_BYTES, dX, lddx, icw, L.kq, m0, M, lane);
    };

    // ---- a wave in a weak half --------------------------------------------------------------------------
    // Fragment t of lane fr is line (channel) 64 lb + 32 t + fr of the half, 16 bytes of it as they are.
    auto run_weak = [&]() {
        uint32_t wrd[4];  // weak lines of fragment 0, indexed by (XOR constant) / 2
#pragma unroll
        for (int x = 0; x < 4; ++x)
            wrd[x] = lds0 + DX_LINE_BASE + (uint32_t)half * DX_HALF + (uint32_t)(64 * lb + fr) * DX_LINE +
                     ((uint32_t)((fk ^ (fr >> 3)) ^ (2 * x)) << 4);
        auto read_a = [&](int set, int i, int buf, int kn) {
            afr[set][i] = *reinterpret_cast<const lds_u4*>(wrd[kn ^ (2 * (i & 1))] + (uint32_t)(i * 32 * DX_LINE + buf * DX_LINES));
        };
#pragma unroll
        for (int j = 0; j < 8; ++j) read_b(0, j, 0, 0);
#pragma unroll
        for (int i = 0; i < 2; ++i) read_a(0, i, 0, 0);

        auto stage = [&](int st, auto cur_c) {
            constexpr int CUR = decltype(cur_c)::value, NXT = CUR ^ 1;
            const int sl = min(st + 2, nst - 1);
            protect();
            asm volatile("" : "+v"(wrd[0]), "+v"(wrd[1]), "+v"(wrd[2]), "+v"(wrd[3]));
            auto step = [&](auto t_c) {
                constexpr int T = decltype(t_c)::value, ks = T >> 4, t = T & 15, kn = (ks + 1) & 3;
                constexpr int SRC = ks < 3 ? CUR : NXT;
                mfma_step(t_c);
                if ((t & 1) == 0) read_b(kn & 1, t >> 1, SRC, kn);
                if (t == 3 || t == 7) read_a(kn & 1, t >> 2, SRC, kn);
                produce_step(t_c, std::integral_constant<int, NXT>{}, sl);
                if (T == 47) __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
            };
            QEFT_STEPS64(step)
        };
        run_stages(stage);
        store_f16_lds_64x256<false>(acc, lds + wave * TILE_BYTES, dX, lddx, icw, L.ic, m0, M, lane);
    };
#undef QEFT_STEPS64
#undef QEFT_STEPS8

    if (H0 == H1) {
        if (H0 == 0) run_quant(); else run_weak();
    } else {
        if (half == 0) run_quant(); else run_weak();
    }
}

// splits > 1: a workgroup (tile, sp) of a split tile contracts over the weight rows [sp * rps, (sp + 1) * rps) only (rps
// a multiple of 64: whole stages) and stores its partial tile as fp16 into its slot of `part`; splitk_reduce_kernel
// adds them.  Which tiles are split: split_tile.  The rows of a stored layer are independent, so a split is simply the
// layer made of those rows.
__device__ __forceinline__ void dx_rega_body(unsigned char* lds, Layer L, const __half* __restrict__ dY, int M, int64_t lddy,
                                             __half* __restrict__ dX, int64_t lddx, int tiles_ic, int splits,
                                             int rps, int tail_first, __half* __restrict__ part) {
    const int tiles_all = tiles_ic * ((M + BT - 1) / BT);
    int tile, sp, slot;
    if (!split_tile(tiles_all, tail_first, splits, tile, sp, slot)) return;
    int t_ic, t_m;
    tile_coords(tile, tiles_ic, (M + BT - 1) / BT, t_ic, t_m);
    const int ic0 = t_ic * BT, m0 = t_m * BT;
    if (slot >= 0) {
        const int r0 = sp * rps;
        L.qweight += (size_t)r0 * L.stride;
        L.scales += (size_t)r0 * L.gs;
        L.zeros += (size_t)r0 * L.gs;
        L.weak += (size_t)r0 * L.k;
        L.oc = min(rps, L.oc - r0);
        dY += r0;
        // the tile stores dX[m][ic] with absolute indices: point it at the slot's (m0, ic0)
        dX = part + (size_t)slot * (BT * BT) - ((size_t)m0 * BT + ic0);
        lddx = BT;
    }
    // a half is weak when it starts at or past Kq (Kq % 128 == 0); without a weak block the surplus
    // half of the last tile runs as a quantized one on clamped addresses and stores nothing
    const bool w0 = L.k > 0 && ic0 >= L.kq, w1 = L.k > 0 && ic0 + 128 >= L.kq;
    if (w0) dx_tile<1, 1>(L, dY, M, lddy, dX, lddx, ic0, m0, lds);
    else if (w1) dx_tile<0, 1>(L, dY, M, lddy, dX, lddx, ic0, m0, lds);
    else dx_tile<0, 0>(L, dY, M, lddy, dX, lddx, ic0, m0, lds);
}
__global__ __launch_bounds__(256) void gemm_dx_rega_kernel(Layer L, const __half* __restrict__ dY, int M, int64_t lddy,
                                                           __half* __restrict__ dX, int64_t lddx, int tiles_ic, int splits,
                                                           int rps, int tail_first, __half* __restrict__ part) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    dx_rega_body(lds, L, dY, M, lddy, dX, lddx, tiles_ic, splits, rps, tail_first, part);
}

// ======================================================================================= weak gradient
// A[i = c][k = m] = Xw[m][c], B[j = oc][k = m] = dY[m][oc]: both operands are read transposed.
// The tokens are split over `splits` workgroups per strip of output channels; each writes an fp32 partial
// [OC][k] slab, summed in slab order by a second kernel (no atomics: deterministic).
// The kernel is sized for what bounds it - reading dY once from
// HBM: a workgroup owns 64 output channels x up to 128 weak columns over a range of tokens, so the
// MFMA tiles hold no padding and a dY row contributes 128 contiguous bytes.  Both operands have
// the contraction index (the token) as their row index; instead of transposing 8 x 8 blocks in
// registers, the tiles go to LDS as they are ([token][column], rows padded by 64 bytes) and the
// fragments are read with the transposing LDS load of gfx950 (ds_read_b64_tr_b16: the 16 lanes
// of a group each name 4 consecutive halfs; output lane l receives element l % 4 of source
// lanes l / 4, l / 4 + 4, l / 4 + 8, l / 4 + 12).  With source lane s pointing at row k0 + s / 4,
// columns c0 + 4 (s % 4) .., a group receives columns c0 .. c0 + 15 of rows k0 .. k0 + 3 - four
// consecutive contraction steps for 16 MFMA rows; two such loads make one fragment.
// Wave w multiplies weak columns 32 w .. 32 w + 31 against the 64 channels.  With one split
// the result goes straight to dW, otherwise into fp32 slabs as above.
constexpr int WG_OC = 64;                             // output channels per workgroup
// Row pitches: a transposing fragment read takes, per half wave, 4 rows x 64 bytes (two 16-lane groups side by
// side), so consecutive rows must sit 16 (or 48) banks apart: 256 + 64 and 128 + 64 bytes.  (With + 32 bytes a
// third of the LDS cycles of this kernel were bank conflicts.)
constexpr int WG_A_PITCH = 128 * 2 + 64;              // bytes per token row of the Xw tile
constexpr int WG_B_PITCH = WG_OC * 2 + 64;            // ... of the dY tile
constexpr int WG_A_BYTES = BK * WG_A_PITCH, WG_B_BYTES = BK * WG_B_PITCH;
constexpr int WG_LDS = 2 * (WG_A_BYTES + WG_B_BYTES); // A0 A1 B0 B1

// A weak block wider than 128 columns is taken in halves of 128 (workgroup index = ((strip, half), split)): the two halves
// of a strip read the same dY rows and sit next to each other in the grid.
// (bid: the workgroup's index among the strip workgroups; lds: its dynamic shared memory, WG_LDS bytes)
__device__ __forceinline__ void weak_grad_strip_body(unsigned char* lds, int bid, int oc_total, int k_total, const __half* __restrict__ dY, int M,
                                                     int64_t lddy, const __half* __restrict__ Xw, int64_t ldxw,
                                                     float* __restrict__ part, int splits, int chunk, void* dW,
                                                     int out_f32, int accumulate) {
    typedef short s4 __attribute__((ext_vector_type(4)));
    typedef short s8 __attribute__((ext_vector_type(8)));
    using lds_s4 = __attribute__((address_space(3))) s4;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int halves = (k_total + 127) >> 7;
    const int split = bid % splits, rest = bid / splits;
    const int kh = rest % halves, t_oc = rest / halves;
    const int k = min(128, k_total - 128 * kh);   // this workgroup's weak columns: 128 kh .. 128 kh + k - 1
    Xw += 128 * kh;
    const int oc0 = t_oc * WG_OC;
    const int mb = split * chunk, me = min(mb + chunk, M);
    const int nst = (me - mb + BK - 1) / BK;
    const int fr = lane & 31, fk = lane >> 5;

    // producers: 16-byte chunks, copied as they are.  Xw tile: 64 tokens x 16 chunks, four per
    // thread (token ar + 16 u, chunk ac); dY tile: 64 tokens x 8 chunks, two per thread (token
    // br + 32 u, chunk bc).  Chunks past k or past the last channel read column 0 and are zeroed.
    const int ar = tid >> 4, ac = tid & 15, br = tid >> 3, bc = tid & 7;
    const bool a_ok = 8 * ac < k, b_ok = oc0 + 8 * bc < oc_total;
    const u4 zero4 = u4{0u, 0u, 0u, 0u};
    // Addresses: a scalar base per stage plus a per-thread byte offset computed once (this kernel is bound by
    // its single wave's instruction stream, and per-load address arithmetic was a third of it).  A stage whose
    // 64 tokens would pass the end of the matrices is fetched 64 tokens back from the end instead (M >= 64) and
    // put() keeps only the rows that belong to it; stages past the range re-read the last one and store zeros.
    using gptr = const __attribute__((address_space(1))) char*;
    using g_u4 = const __attribute__((address_space(1))) u4;
    uint32_t aoff[4], boff[2];
#pragma unroll
    for (int u = 0; u < 4; ++u) aoff[u] = (uint32_t)(((int64_t)(ar + 16 * u) * ldxw + (a_ok ? 8 * ac : 0)) * 2);
#pragma unroll
    for (int u = 0; u < 2; ++u) boff[u] = (uint32_t)(((int64_t)(br + 32 * u) * lddy + (b_ok ? oc0 + 8 * bc : 0)) * 2);
    const bool cols_full = __builtin_amdgcn_readfirstlane((int)(k >= 8 * 16 && oc0 + WG_OC <= oc_total)) != 0;   // no thread's chunk is zeroed
    auto first_token = [&](int st) { return min(mb + BK * min(st, nst - 1), M - BK); };   // of the 64 tokens fetched for stage st
    // three stages of fetches in flight per thread (registers), a fourth in LDS being multiplied
    u4 va[3][4], vb[3][2];
    auto fetch = [&](auto set_c, int st) {
        constexpr int SET = decltype(set_c)::value;
        const int t0 = first_token(st);
        const char* ab = reinterpret_cast<const char*>(Xw) + (int64_t)t0 * ldxw * 2;
        const char* bb = reinterpret_cast<const char*>(dY) + (int64_t)t0 * lddy * 2;
        asm volatile("" : "+s"(ab), "+s"(bb));
#pragma unroll
        for (int u = 0; u < 4; ++u) va[SET][u] = *reinterpret_cast<g_u4*>((gptr)ab + aoff[u]);
#pragma unroll
        for (int u = 0; u < 2; ++u) vb[SET][u] = *reinterpret_cast<g_u4*>((gptr)bb + boff[u]);
    };
    auto put = [&](auto set_c, int st, int buf) {   // stage st, held by register set SET, into LDS buffer buf
        constexpr int SET = decltype(set_c)::value;
        const int m0 = mb + BK * st, t0 = first_token(st);
        unsigned char* sA = lds + buf * WG_A_BYTES;
        unsigned char* sB = lds + 2 * WG_A_BYTES + buf * WG_B_BYTES;
        if (cols_full && st < nst && m0 + BK <= me) {   // a whole stage, whole columns (wave-uniform): the registers as they are
#pragma unroll
            for (int u = 0; u < 4; ++u) *reinterpret_cast<u4*>(sA + (ar + 16 * u) * WG_A_PITCH + 16 * ac) = va[SET][u];
#pragma unroll
            for (int u = 0; u < 2; ++u) *reinterpret_cast<u4*>(sB + (br + 32 * u) * WG_B_PITCH + 16 * bc) = vb[SET][u];
        } else if (st >= nst) {   // past the range: a tile of zeros
#pragma unroll
            for (int u = 0; u < 4; ++u) *reinterpret_cast<u4*>(sA + (ar + 16 * u) * WG_A_PITCH + 16 * ac) = zero4;
#pragma unroll
            for (int u = 0; u < 2; ++u) *reinterpret_cast<u4*>(sB + (br + 32 * u) * WG_B_PITCH + 16 * bc) = zero4;
        } else {
            // fetched row r holds token t0 + r; it belongs to the stage when that lies in [m0, me), and its tile row
            // is token - m0.  shift = m0 - t0 > 0 only for the last stage of the matrices: fetched rows [shift, 64)
            // fill tile rows [0, 64 - shift), the rest of the tile is zero.
            const int shift = m0 - t0;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int r = ar + 16 * u, tok = t0 + r;
                if (r >= shift) *reinterpret_cast<u4*>(sA + (r - shift) * WG_A_PITCH + 16 * ac) = (a_ok && tok < me) ? va[SET][u] : zero4;
                if (r >= BK - shift) *reinterpret_cast<u4*>(sA + r * WG_A_PITCH + 16 * ac) = zero4;
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int r = br + 32 * u, tok = t0 + r;
                if (r >= shift) *reinterpret_cast<u4*>(sB + (r - shift) * WG_B_PITCH + 16 * bc) = (b_ok && tok < me) ? vb[SET][u] : zero4;
                if (r >= BK - shift) *reinterpret_cast<u4*>(sB + r * WG_B_PITCH + 16 * bc) = zero4;
            }
        }
    };

    f16v acc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;

    // fragment addressing: lane = 16 g + s; rows (tokens) 8 (g / 2) + s / 4 (+ 4 for the second
    // load, + 16 per k-block), columns 16 (g % 2) + 4 (s % 4) of the wave's 32
    const int g = lane >> 4, s = lane & 15;
    const int frow = 8 * (g >> 1) + (s >> 2), fcol = 16 * (g & 1) + 4 * (s & 3);
    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char*)lds;
    const uint32_t fa = lds0 + frow * WG_A_PITCH + 2 * (32 * wave + fcol);
    const uint32_t fb = lds0 + 2 * WG_A_BYTES + frow * WG_B_PITCH + 2 * fcol;
    auto frag = [&](uint32_t addr, int pitch) {   // 8 contraction steps: rows +0..3 and +4..7
        const s4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)(size_t)(addr));
        const s4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)(size_t)(addr + 4 * pitch));
        return __builtin_bit_cast(h8, s8{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w});
    };

    // stage st (already in LDS buffer st & 1, fetched through register set SET): refill the set
    // with stage st + 3, multiply, move stage st + 1 from the next set into the other buffer
    auto stage = [&](auto set_c, int st) {
        constexpr int SET = decltype(set_c)::value;
        const int cur = st & 1;
        fetch(set_c, st + 3);
        __builtin_amdgcn_sched_barrier(0);   // issue the fetches first: they are what the stage waits for
        const uint32_t a0 = fa + cur * WG_A_BYTES, b0 = fb + cur * WG_B_BYTES;
        // fragments are read one k-block ahead of the MFMAs that use them (one wave per SIMD: nothing else hides the LDS latency)
        h8 a[2], bl[2], bh[2];
        auto frags = [&](int ks) {
            a[ks & 1] = frag(a0 + 16 * ks * WG_A_PITCH, WG_A_PITCH);
            bl[ks & 1] = frag(b0 + 16 * ks * WG_B_PITCH, WG_B_PITCH);
            bh[ks & 1] = frag(b0 + 16 * ks * WG_B_PITCH + 64, WG_B_PITCH);
        };
        frags(0);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks < 3) frags(ks + 1);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[ks & 1], bl[ks & 1], acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[ks & 1], bh[ks & 1], acc[1], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        put(std::integral_constant<int, (SET + 1) % 3>{}, st + 1, cur ^ 1);
        __syncthreads();
    };
    fetch(std::integral_constant<int, 0>{}, 0);
    fetch(std::integral_constant<int, 1>{}, 1);
    fetch(std::integral_constant<int, 2>{}, 2);
    put(std::integral_constant<int, 0>{}, 0, 0);
    __syncthreads();
    // always three stages per turn, with no branch between them (the compiler's wait counting then
    // lets two stages of fetches stay in flight); stages past the range multiply zeros
    for (int st = 0; st < nst; st += 3) {
        stage(std::integral_constant<int, 0>{}, st);
        stage(std::integral_constant<int, 1>{}, st + 1);
        stage(std::integral_constant<int, 2>{}, st + 2);
    }
    if (32 * wave >= k) return;   // this wave's weak columns do not exist
    // lane (fr, fk) holds, for channel oc0 + 32 t + fr, weak columns 32 wave + 8 g + 4 fk .. + 3
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int j = oc0 + 32 * t + fr;
        if (j >= oc_total) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int i = 32 * wave + 8 * q + 4 * fk;
            if (i >= k) continue;
            f4 r = f4{acc[t][4 * q + 0], acc[t][4 * q + 1], acc[t][4 * q + 2], acc[t][4 * q + 3]};
            const size_t at = (size_t)j * k_total + 128 * kh + i;
            if (splits > 1) {
                *reinterpret_cast<f4*>(part + (size_t)split * oc_total * k_total + at) = r;
            } else if (out_f32) {
                f4* o = reinterpret_cast<f4*>((float*)dW + at);
                *o = accumulate ? *o + r : r;
            } else {
                __half* o = (__half*)dW + at;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = __float2half_rn(accumulate ? __half2float(o[e]) + r[e] : r[e]);
            }
        }
    }
}

__global__ __launch_bounds__(256) void weak_grad_strip_kernel(int oc_total, int k_total, const __half* __restrict__ dY, int M,
                                                              int64_t lddy, const __half* __restrict__ Xw, int64_t ldxw,
                                                              float* __restrict__ part, int splits, int chunk, void* dW,
                                                              int out_f32, int accumulate) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    weak_grad_strip_body(lds, (int)blockIdx.x, oc_total, k_total, dY, M, lddy, Xw, ldxw, part, splits, chunk, dW, out_f32, accumulate);
}

// The input gradient and the weak block's gradient of one layer in ONE launch: the first n_dx workgroups are the
// tiles of gemm_dx_rega_kernel (no split), the rest the strips of weak_grad_strip_kernel.  Both read dY; the
// strips are dispatched as compute units fall free, i.e. into the partly empty last round of tiles (688 tiles on
// 256 units leave 80 of them idle for a third of the launch), where they cost nothing.
__global__ __launch_bounds__(256) void gemm_dx_dw_kernel(Layer L, const __half* __restrict__ dY, int M, int64_t lddy,
                                                         __half* __restrict__ dX, int64_t lddx, int tiles_ic, int n_dx,
                                                         const __half* __restrict__ Xw, int64_t ldxw, float* __restrict__ part,
                                                         int splits, int chunk, void* dW, int out_f32, int accumulate) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    if ((int)blockIdx.x >= n_dx) {
        weak_grad_strip_body(lds, (int)blockIdx.x - n_dx, L.oc, L.k, dY, M, lddy, Xw, ldxw, part, splits, chunk, dW, out_f32, accumulate);
        return;
    }
    dx_rega_body(lds, L, dY, M, lddy, dX, lddx, tiles_ic, 1, 0, 0, nullptr);
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

}  // namespace

// The tiled kernels round every dequantized weight once to fp16 (relative 2^-11).  Over a long contraction these
// roundings average out far below the parity bar; a sum of a handful of terms has no such averaging and single
// outputs can leave the per-element bar, so contractions shorter than 64 terms (IC here, OC for the input
// gradient) take the general kernels, which keep s (q - z) in fp32.
constexpr int MIN_CONTRACTION = 64;

bool gemm_fwd_supported(const Layer& L, int64_t M) {
    return M >= 1 && L.bits == 4 && L.g == 128 && (L.kq % 8) == 0 && (L.k % 8) == 0 && (L.oc % 8) == 0 && L.ic >= MIN_CONTRACTION;
}

namespace {
// Sum of the partial tiles of the split tiles: workgroup (tail index, r) adds the `splits` slots of rows 8 r .. 8 r + 7
// of one tile, 8 outputs (16 bytes) per thread, fp32 sum in split order, one rounding.  n: columns of the output
// (tiles_n tiles of them).
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const __half* __restrict__ part, int splits, int tiles_all, int tiles_n,
                                                            int tail_first, int M, int n, __half* __restrict__ Y, int64_t ldy) {
    const int tt = blockIdx.x >> 5, part32 = blockIdx.x & 31;
    const int tile = split_tail_tile(tiles_all, tail_first, tt);
    if (tile < 0) return;
    int t_n, t_m;
    tile_coords(tile, tiles_n, (M + BT - 1) / BT, t_n, t_m);
    const int n0 = t_n * BT, m0 = t_m * BT;
    const bool wide = (ldy & 7) == 0 && (reinterpret_cast<uintptr_t>(Y) & 15) == 0;
    const __half* p0 = part + (size_t)tt * splits * (BT * BT);
    {
        const int row = part32 * 8 + (threadIdx.x >> 5), c = threadIdx.x & 31;
        const int m = m0 + row, col = n0 + 8 * c;
        if (m >= M || col >= n) return;
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
        for (int p = 0; p < splits; ++p) {
            const u4 v = ld16(p0 + (size_t)p * (BT * BT) + row * BT + 8 * c);
            const h8 h = __builtin_bit_cast(h8, v);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += (float)h[e];
        }
        __half* y = Y + (size_t)m * ldy + col;
        if (col + 8 <= n && wide) {
            h8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (_Float16)acc[e];
            *reinterpret_cast<u4*>(y) = __builtin_bit_cast(u4, o);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (col + e < n) y[e] = __float2half_rn(acc[e]);
        }
    }
}

// Which tiles to split and how, for a launch of `tiles` tiles whose contraction has `chunks` units of 8 stages.
//   fewer than 160 tiles: all of them, as many ways as bring the workgroups to about the number of CUs (at most 16);
//   otherwise the tiles of each XCD's last round when that round fills at most half of the XCD's 32 CUs, as many ways as
//   fill it (at most 8) - provided the time saved on that round (stage_us per stage) is well above the cost of the
//   partial tiles' traffic and the second launch.
struct SplitPlan {
    int splits = 1, chunks_per_split = 0, tail_first = 0;
};
SplitPlan plan_split(int tiles, int stages) {
    SplitPlan p;
    const int chunks = stages / 8;
    if (chunks < 2) return p;
    int want;
    if (tiles < 160) {
        want = 256 / tiles;
        want = want > 16 ? 16 : want;
    } else {
        const int per = ceil_div(tiles, N_XCD), full = per / 32 * 32, rem = per - full;
        if (rem == 0 || rem > 16 || full == 0) return p;
        want = 32 / rem;
        want = want > 8 ? 8 : want;
        p.tail_first = full;
    }
    const int chunks_all = ceil_div(stages, 8);   // a ragged last chunk included
    want = want > chunks_all ? chunks_all : want;
    if (want < 2) return SplitPlan();
    p.chunks_per_split = ceil_div(chunks_all, want);   // at most `want` splits
    p.splits = ceil_div(stages, p.chunks_per_split * 8);
    if (p.splits < 2) return SplitPlan();
    if (p.tail_first > 0) {
        // measured: a stage takes 1.6 - 1.8 us with every CU busy; the second launch 7 - 9 us for 256 slots
        const double saved = (stages - p.chunks_per_split * 8) * 1.6;                                // us
        const double cost = 8.0 + split_tail_tiles(tiles, p.tail_first) * p.splits * 0.05;           // us: 128 KB written and read per slot
        if (saved < 1.5 * cost) return SplitPlan();
    }
    return p;
}
size_t split_workspace(int tiles, const SplitPlan& p) {
    return p.splits > 1 ? (size_t)split_tail_tiles(tiles, p.tail_first) * p.splits * BT * BT * sizeof(__half) : 0;
}
}  // namespace

// K split of the forward: units of 8 stages (512 columns)
static SplitPlan gemm_fwd_plan(const Layer& L, int64_t M) {
    const int tiles = ceil_div(L.oc, BT) * ceil_div(M, BT);
    if (L.kq == 0 && L.k > 0 && L.k % BK == 0) return plan_split(tiles, L.k / BK);   // all fp16: the weak stages are split
    if (L.kq <= 0 || L.kq % BK != 0) return SplitPlan();
    return plan_split(tiles, L.kq / BK);
}

size_t gemm_fwd_split_workspace(const Layer& L, int64_t M) {
    return split_workspace(ceil_div(L.oc, BT) * ceil_div(M, BT), gemm_fwd_plan(L, M));
}

hipError_t gemm_fwd(const Layer& L, const __half* X, int64_t M, int64_t ldx, __half* Y, int64_t ldy, void* ws, hipStream_t s) {
    const int tiles_oc = ceil_div(L.oc, BT), tiles_m = ceil_div(M, BT);
    hipError_t e;
    if (L.kq % BK == 0 && (L.kq > 0 || (L.k > 0 && L.k % BK == 0))) {   // whole stages: weights straight into MFMA operand registers
        static bool attr = false;
        if (!attr) {
            e = hipFuncSetAttribute((const void*)gemm_fwd_rega_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, REGA_LDS);
            if (e != hipSuccess) return e;
            attr = true;
        }
        const int tiles = tiles_oc * tiles_m;
        const int wide = (ldy % 8 == 0) && (reinterpret_cast<uintptr_t>(Y) % 16 == 0);
        const SplitPlan p = ws ? gemm_fwd_plan(L, M) : SplitPlan();
        if (p.splits > 1) {
            __half* part = (__half*)ws;
            gemm_fwd_rega_kernel<<<split_grid(tiles, p.tail_first, p.splits), 256, REGA_LDS, s>>>(L, X, (int)M, ldx, Y, ldy, tiles_oc, wide, p.splits,
                                                                                                 p.chunks_per_split * 8, p.tail_first, part);
            splitk_reduce_kernel<<<32 * split_tail_tiles(tiles, p.tail_first), 256, 0, s>>>(part, p.splits, tiles, tiles_oc, p.tail_first, (int)M,
                                                                                           L.oc, Y, ldy);
            return hipGetLastError();
        }
        gemm_fwd_rega_kernel<<<xcd_grid(tiles), 256, REGA_LDS, s>>>(L, X, (int)M, ldx, Y, ldy, tiles_oc, wide, 1, 0, 0, nullptr);
    } else {
        static bool attr = false;
        e = raise_lds_limit((const void*)gemm_fwd_kernel, attr);
        if (e != hipSuccess) return e;
        gemm_fwd_kernel<<<xcd_grid(tiles_oc * tiles_m), 256, GEMM_LDS, s>>>(L, X, (int)M, ldx, Y, ldy, tiles_oc);
    }
    return hipGetLastError();
}

bool gemm_dx_supported(const Layer& L, int64_t M) {
    return M > 16 && L.bits == 4 && L.g == 128 && (L.kq % 8) == 0 && (L.k % 8) == 0 && (L.oc % 8) == 0 &&
           (L.ic % 8) == 0 && L.oc >= MIN_CONTRACTION;
}

// Row split of the input gradient, as for the forward: units of 8 stages (512 rows).
static SplitPlan gemm_dx_plan(const Layer& L, int64_t M) {
    if (!(L.oc % BK == 0 && L.kq % 128 == 0 && L.k % 8 == 0)) return SplitPlan();
    return plan_split(ceil_div(L.ic, BT) * ceil_div(M, BT), L.oc / BK);
}

size_t gemm_dx_split_workspace(const Layer& L, int64_t M) {
    return split_workspace(ceil_div(L.ic, BT) * ceil_div(M, BT), gemm_dx_plan(L, M));
}

hipError_t gemm_dx(const Layer& L, const __half* dY, int64_t M, int64_t lddy, __half* dX, int64_t lddx, void* ws, hipStream_t s) {
    const int tiles_m = ceil_div(M, BT), tiles_ic = ceil_div(L.ic, BT);
    hipError_t e;
    if (L.oc % BK == 0 && L.kq % 128 == 0 && L.k % 8 == 0) {
        static bool attr = false;
        if (!attr) {
            e = hipFuncSetAttribute((const void*)gemm_dx_rega_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, DX_LDS);
            if (e != hipSuccess) return e;
            attr = true;
        }
        const int tiles = tiles_ic * tiles_m;
        const SplitPlan p = ws ? gemm_dx_plan(L, M) : SplitPlan();
        if (p.splits > 1) {
            __half* part = (__half*)ws;
            gemm_dx_rega_kernel<<<split_grid(tiles, p.tail_first, p.splits), 256, DX_LDS, s>>>(L, dY, (int)M, lddy, dX, lddx, tiles_ic, p.splits,
                                                                                              p.chunks_per_split * 8 * BK, p.tail_first, part);
            splitk_reduce_kernel<<<32 * split_tail_tiles(tiles, p.tail_first), 256, 0, s>>>(part, p.splits, tiles, tiles_ic, p.tail_first, (int)M,
                                                                                           L.ic, dX, lddx);
            return hipGetLastError();
        }
        gemm_dx_rega_kernel<<<xcd_grid(tiles), 256, DX_LDS, s>>>(L, dY, (int)M, lddy, dX, lddx, tiles_ic, 1, 0, 0, nullptr);
    } else {
        static bool attr = false;
        e = raise_lds_limit((const void*)gemm_dx_kernel, attr);
        if (e != hipSuccess) return e;
        gemm_dx_kernel<<<xcd_grid(tiles_ic * tiles_m), 256, GEMM_LDS, s>>>(L, dY, (int)M, lddy, dX, lddx, tiles_ic, 0);
    }
    return hipGetLastError();
}

bool weak_grad_mfma_supported(int oc, int k, int64_t M) {
    return M >= 64 && k >= 8 && k <= BT && (k % 8) == 0 && (oc % 8) == 0;
}

namespace {
// split of the tokens for the strip kernel: about one workgroup per CU (more splits would add
// slab traffic comparable to dY itself), every split a whole number of stages
void weak_grad_strip_split(int oc, int k, int64_t M, int& splits, int& chunk) {
    const int tiles = ceil_div(oc, WG_OC) * ceil_div(k, 128);
    const int stages = ceil_div(M, BK);
    int want = ceil_div(256, tiles);
    if (want > stages) want = stages;
    if (want < 1) want = 1;
    chunk = ceil_div(stages, want) * BK;
    splits = ceil_div(M, chunk);
}
}  // namespace

size_t weak_grad_mfma_workspace(int oc, int k, int64_t M) {
    int splits, chunk;
    weak_grad_strip_split(oc, k, M, splits, chunk);
    return splits > 1 ? (size_t)splits * oc * k * sizeof(float) : 0;
}

hipError_t weak_grad_mfma(int oc, int k, const __half* dY, int64_t M, int64_t lddy, const __half* Xw, int64_t ldxw,
                          void* dW, int out_f32, int accumulate, void* ws, hipStream_t s) {
    int splits, chunk;
    const int64_t n = (int64_t)oc * k;
    weak_grad_strip_split(oc, k, M, splits, chunk);
    static bool strip_attr = false;
    if (!strip_attr) {
        hipError_t e = hipFuncSetAttribute((const void*)weak_grad_strip_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, WG_LDS);
        if (e != hipSuccess) return e;
        strip_attr = true;
    }
    weak_grad_strip_kernel<<<ceil_div(oc, WG_OC) * ceil_div(k, 128) * splits, 256, WG_LDS, s>>>(oc, k, dY, (int)M, lddy, Xw, ldxw, (float*)ws, splits,
                                                                                          chunk, dW, out_f32, accumulate);
    if (splits > 1) weak_grad_reduce_kernel<<<ceil_div(n, 256), 256, 0, s>>>((const float*)ws, splits, n, dW, out_f32, accumulate);
    return hipGetLastError();
}

// dX and dW_weak of one layer in one launch (see gemm_dx_dw_kernel); false when the shapes do not fit both
// register kernels (the caller then makes the two calls one after the other).
// Taken when the weak block is one strip wide (k <= 128).  The strips follow the tiles in the grid, so they start on
// whichever compute units finish their last tile first: in the idle part of a partly empty last round, or, when the
// tiles fill their rounds, in the few microseconds by which the tiles' ends differ.  Inside the combined launch a strip
// workgroup has a compute unit to itself (the launch reserves the tile kernel's LDS and registers for every workgroup;
// on its own the strip kernel runs two per unit), so a weak gradient that is heavy next to that idle time loses more
// than it gains.  Measured at M = 4096, the two calls against the one: 11008 x 4096 (256 tiles) 388 -> 382 us,
// 4096 x 4096 (256 tiles) 165 -> 163, 4096 x 11008 (688 tiles) 363 -> 350, 5120 x 5120 281 -> 262, 13824 x 5120
// 699 -> 670; with a 256-wide weak block (two half strips per strip of channels) 8192 x 8192 at M = 2048 257 -> 252
// but 28672 x 8192 862 -> 877.
bool gemm_dx_dw_supported(const Layer& L, int64_t M) {
    return gemm_dx_supported(L, M) && L.oc % BK == 0 && L.kq % 128 == 0 && L.k % 8 == 0 && L.k > 0 && L.k <= 128 &&
           weak_grad_mfma_supported(L.oc, L.k, M);
}

hipError_t gemm_dx_dw(const Layer& L, const __half* dY, int64_t M, int64_t lddy, __half* dX, int64_t lddx, const __half* Xw,
                      int64_t ldxw, void* dW, int out_f32, int accumulate, void* ws, hipStream_t s) {
    const int tiles = ceil_div(L.ic, BT) * ceil_div(M, BT), n_dx = xcd_grid(tiles);
    int splits, chunk;
    const int64_t n = (int64_t)L.oc * L.k;
    weak_grad_strip_split(L.oc, L.k, M, splits, chunk);
    static bool attr = false;
    constexpr int LDS_BYTES = DX_LDS > WG_LDS ? DX_LDS : WG_LDS;
    if (!attr) {
        hipError_t e = hipFuncSetAttribute((const void*)gemm_dx_dw_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        attr = true;
    }
    const int n_dw = ceil_div(L.oc, WG_OC) * ceil_div(L.k, 128) * splits;
    gemm_dx_dw_kernel<<<n_dx + n_dw, 256, LDS_BYTES, s>>>(L, dY, (int)M, lddy, dX, lddx, ceil_div(L.ic, BT), n_dx, Xw, ldxw, (float*)ws, splits,
                                                         chunk, dW, out_f32, accumulate);
    if (splits > 1) weak_grad_reduce_kernel<<<ceil_div(n, 256), 256, 0, s>>>((const float*)ws, splits, n, dW, out_f32, accumulate);
    return hipGetLastError();
}

}  // namespace qeft
