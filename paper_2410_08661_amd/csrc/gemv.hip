// Decode path (paper Sec. 3.2.1): Y = X . W^T for M <= 16 rows in one fused pass over the
// packed 4-bit codes, the group parameters and the fp16 weak block.  HBM-bound: the kernel
// streams every stored byte exactly once with 128-bit loads.
//
// Mapping.  The product runs on the 16x16x32 fp16 MFMA with the M (<= 16, zero padded)
// activation rows as the A operand and 16 output channels as the B operand.  In that
// instruction lane l supplies 8 contraction elements of row/column l % 16 for the slot
// l / 16, and one packed 32-bit word holds exactly 8 codes: a lane's 128-bit load (4 words
// = 32 codes) therefore feeds 4 MFMAs with no cross-lane movement, and the 4 slots of a
// load cover 128 consecutive columns = one quantization group ("step").  Which column a
// contraction slot stands for is free as long as A and B agree, so the activations are
// permuted to the order the nibbles come out of the mask-and-or conversion
// (pairs (0,4) (1,5) (2,6) (3,7)).
//
// Dequantization never touches the weights: the codes enter the MFMA as the exact fp16
// numbers 1024 + q (exponent bits or-ed onto the nibble) and the group's contribution is
//     s * (sum x*(1024+q) - (1024 + z) * Sx) = s * sum x*(q - z),   Sx = sum of the group's x,
// applied to the 16x16 fp32 accumulator: 2 FMAs per 32 weights and lane, any fp16 zero-point.
// The weak block is a plain fp16 B operand accumulated into the same tile.
//
// Work split.  A workgroup owns whole tiles of 16 output channels; KS waves per tile split
// the K steps into contiguous ranges and are reduced through LDS in a fixed order (no
// atomics: run-to-run deterministic).  Weight loads run several steps ahead in loops without
// branches (rows are padded to whole steps and rows past OC are clamped, never stored).
//   * small-M kernel (M <= 4 and X fits in LDS; today M = 2, M = 3 and 4 on rows of several passes, and the dense
//     3-bit layout at 2 <= M <= 4): the workgroup stages X once (permuted, with
//     Sx), one barrier; a launch-latency-shaped prologue (see the kernel).  It also takes a
//     group of layers that share X (query / key / value, gate / up) as one launch: its tiles
//     are those of layer 0, then layer 1, ..., each wave picking its layer's pointers;
//   * register kernel (5 <= M <= 16; M = 3 and 4 on rows of a single pass): one wave per K range keeps the A
//     fragments of its range in registers for the whole launch (no workgroup staging, no barrier before the
//     stream), walks several row tiles and meets the other waves' partial tiles in LDS at the end;
//   * one activation row goes to a kernel of its own (gemv_dot.hip): whole rows per wave, two-element dot
//     products, activations in registers;
//   * row-batch kernel (any M <= 16): nothing staged, A fragments straight from X, Sx from the
//     matrix core (fallback for shapes the register kernel does not take);
//   * 3-bit kernel (any M <= 16): weight-side dequantization, ten codes per word;
//   * chunked kernel: each wave stages its own slice, CH steps at a time (fallback only).
//
// Every branch around an MFMA is wave-uniform by construction (the wave index goes through
// readfirstlane): MFMA executes regardless of the EXEC mask.
#include <cstdlib>
#include <type_traits>

#include <climits>
#include "qeft_internal.h"

namespace qeft {
namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ h8 as_h8(u4 v) { return __builtin_bit_cast(h8, v); }
__device__ __forceinline__ u4 load16(const void* p) { return *reinterpret_cast<const u4*>(p); }
__device__ __forceinline__ u2 load8(const void* p) { return *reinterpret_cast<const u2*>(p); }
// element i (0..3) of four packed halfs
__device__ __forceinline__ float half_at(u2 v, int i) { return (float)__builtin_bit_cast(h2, (i < 2) ? v.x : v.y)[i & 1]; }

// The two constants of the code -> fp16 conversion, held in vector registers the compiler
// cannot see through: (w & mask) | magic then selects the single v_and_or_b32 (with two
// literals it would be two instructions).  The instruction itself is compiler-generated on
// purpose: VALU instructions hidden in inline asm escape the MFMA hazard recognizer.
struct Consts {
    uint32_t mask, magic;
};
__device__ __forceinline__ Consts make_consts(uint32_t mask = 0x000f000fu) {
    Consts c{mask, 0x64006400u};
    asm volatile("" : "+v"(c.mask), "+v"(c.magic));
    return c;
}

// 8 codes of one word as fp16 (1024 + q), in slot order (0,4)(1,5)(2,6)(3,7)
__device__ __forceinline__ h8 codes_to_h8(uint32_t w, Consts c) {
    u4 r;
    r.x = (w & c.mask) | c.magic;
    r.y = ((w >> 4) & c.mask) | c.magic;
    r.z = ((w >> 8) & c.mask) | c.magic;
    r.w = ((w >> 12) & c.mask) | c.magic;
    return as_h8(r);
}

// 8 consecutive activations (x0..x7 in 4 registers) to the same slot order
__device__ __forceinline__ u4 permute_x(u4 v) {
    u4 r;
    r.x = __builtin_amdgcn_perm(v.z, v.x, 0x05040100u);  // (x0, x4)
    r.y = __builtin_amdgcn_perm(v.z, v.x, 0x07060302u);  // (x1, x5)
    r.z = __builtin_amdgcn_perm(v.w, v.y, 0x05040100u);  // (x2, x6)
    r.w = __builtin_amdgcn_perm(v.w, v.y, 0x07060302u);  // (x3, x7)
    return r;
}

// x0 + ... + x7 in fp32
__device__ __forceinline__ float sum8(u4 v) {
    const h8 h = as_h8(v);
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += (float)h[i];
    return s;
}

// sum over each aligned group of 16 lanes, in every lane of the group: butterfly of four
// data-parallel-primitive moves (lane ^ 1, lane ^ 2, mirrored halves, mirrored row), no LDS round trips
__device__ __forceinline__ float sum16(float t) {
    auto dpp = [](float v, auto ctrl) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), decltype(ctrl)::value, 0xf, 0xf, false));
    };
    t += dpp(t, std::integral_constant<int, 0xB1>{});    // quad_perm [1,0,3,2]
    t += dpp(t, std::integral_constant<int, 0x4E>{});    // quad_perm [2,3,0,1]
    t += dpp(t, std::integral_constant<int, 0x141>{});   // row_half_mirror
    t += dpp(t, std::integral_constant<int, 0x140>{});   // row_mirror
    return t;
}

__device__ __forceinline__ void wave_lds_fence() { __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); }

// Dense 3-bit layout: the lane's 32 codes are the 96 bits w.x, w.y, w.z; octet I is its fragment I, pair P
// of the 16 sits at bits 6 P .. 6 P + 5 (two pairs straddle words).  One field extract, one multiplication
// by 2^13 + 1 (second code to bit 16) and the and-or give the fp16 pair (1024 + q0, 1024 + q1), in column order.
template <int I>
__device__ __forceinline__ h8 dense3_to_h8(u4 w, Consts c) {
    u4 r;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int P = 4 * I + p, wi = (6 * P) >> 5, sh = (6 * P) & 31;
        const uint32_t six = sh <= 26 ? __builtin_amdgcn_ubfe(w[wi], sh, 6)
                                      : __builtin_amdgcn_ubfe(__builtin_amdgcn_alignbit(w[(wi + 1) & 3], w[wi], sh), 0, 6);
        r[p] = ((six * 0x2001u) & c.mask) | c.magic;
    }
    return as_h8(r);
}

// One quantized step of one 16-row tile: 4 MFMAs on the codes, then the group's scale and
// zero-point on the accumulator.  c = 1024 + z.
template <bool W3 = false>
__device__ __forceinline__ void step_tile(f4& y, const u4 (&xa)[4], u4 w, f4 sx, float sf, float c, Consts magic) {
    f4 acc = f4{0.f, 0.f, 0.f, 0.f};
    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(xa[0]), W3 ? dense3_to_h8<0>(w, magic) : codes_to_h8(w.x, magic), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(xa[1]), W3 ? dense3_to_h8<1>(w, magic) : codes_to_h8(w.y, magic), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(xa[2]), W3 ? dense3_to_h8<2>(w, magic) : codes_to_h8(w.z, magic), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(xa[3]), W3 ? dense3_to_h8<3>(w, magic) : codes_to_h8(w.w, magic), acc, 0, 0, 0);
#pragma unroll
    for (int e = 0; e < 4; ++e) y[e] = fmaf(sf, fmaf(-c, sx[e], acc[e]), y[e]);
}

// Weak steps of 32 fp16 columns, dealt to the K-split waves from the last one back (they carry
// fewer quantized steps when the split is uneven).
template <int R>
__device__ __forceinline__ void weak_steps(const Layer& L, const __half* __restrict__ X, int M, int64_t ldx, int row0,
                                           int kw, int KS, int n, int kb, f4 (&y)[R]) {
    const u4 zero4 = u4{0u, 0u, 0u, 0u};
    const int nweak = (L.k + 31) / 32;
    for (int t = KS - 1 - kw; t < nweak; t += KS) {
        const int c0 = 32 * t + 8 * kb;
        const u4 xa = (n < M && c0 < L.k) ? load16(X + (size_t)n * ldx + L.kq + c0) : zero4;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int o = min(row0 + 16 * r + n, L.oc - 1);
            const u4 wk = (c0 < L.k) ? load16(L.weak + (size_t)o * L.k + c0) : zero4;
            y[r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(xa), as_h8(wk), y[r], 0, 0, 0);
        }
    }
}

// Reduction over the K split and store.  `slot(w)` is a float[R*4*64] buffer of K-split wave w.
template <int R, class Slot>
__device__ __forceinline__ void reduce_store(const Layer& L, f4 (&y)[R], int kw, int KS, int lane, int row0, int M,
                                             __half* __restrict__ Y, int64_t ldy, Slot slot) {
    const int n = lane & 15, kb = lane >> 4;
    if (kw > 0) {
        float* mine = slot(kw);
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < 4; ++e) mine[(r * 4 + e) * 64 + lane] = y[r][e];
    }
    __syncthreads();
    if (kw == 0) {
        for (int w = 1; w < KS; ++w) {
            const float* other = slot(w);
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int e = 0; e < 4; ++e) y[r][e] += other[(r * 4 + e) * 64 + lane];
        }
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

// =============================================================================================
// Small-M kernel: M <= 4.  A workgroup owns TW tiles of 16 rows; its TW*KS waves stage all of X
// once (one barrier), then wave (t, kw) streams K range kw of tile t (K split in units of 4 steps).
//
// At these sizes a launch lives for a few microseconds and is bound by memory latency and by the
// number of cache-line requests queued at its start, not by bandwidth, so the prologue is built
// around the request stream:
//   * every request goes out first, in straight-line code - indices are clamped instead of
//     tested, because a load under a branch makes the compiler wait for all outstanding loads at
//     the join, and loads return in order;
//   * X (L2 hits) and the group parameters are requested ahead of the weights, so staging them
//     never waits for HBM; the weights of up to D steps per lane follow at once;
//   * the scales / zero-points of a tile are fetched once per tile, not per K-split wave: chunk c
//     = 32 groups of one array for the tile's 16 rows, one 16-byte load per lane (16 cache lines
//     per request, each used in full), dealt round-robin to the tile's waves, NSZ per wave;
//   * the weak block's loads are exactly the WMAX = ceil(steps / KS) the wave consumes.
// LDS: X [M][ng*256 + 16 B] permuted fragments | Sx float [ng][4] | zero bytes |
//      (s, 1024+z) float2 [tiles][groups][16] | reduction slots
// =============================================================================================
struct SmallLds {
    int xrow, sx_off, zero_off, sz_off, sz_tile, red_off, total, tw;
};
inline SmallLds small_lds(int M, int ng, int tw, int ks) {
    SmallLds l;
    l.xrow = ng * 256 + 16;
    l.sx_off = M * l.xrow;
    l.zero_off = l.sx_off + ng * 16;  // what lanes without an activation row read, D steps deep
    l.sz_off = l.zero_off + 256 * 8;
    l.sz_tile = ng * 128;
    l.red_off = l.sz_off + tw * l.sz_tile;
    l.total = l.red_off + (ks - 1) * tw * 4 * 64 * (int)sizeof(float);
    l.tw = tw;
    return l;
}

// PERM: the activations are in the layer's ORIGINAL channel order and stored column j reads
// X[perm[j]] (weak columns left at arbitrary channels): the 16-byte fragment loads become eight
// 2-byte gathers through the table, whose own requests head the stream.
// W3: 3-bit codes in the dense layout.  A lane's 12 bytes hold the 32 codes of its quarter of a group, so the
// kernel is the same step for step (one group per step, 48 bytes of a row); the activations stay in column
// order, which is the order the 3-bit conversion produces.
template <int D, int WMAX, int NSZ, bool PERM, bool W3 = false>
__global__ __launch_bounds__(1024) void gemv_w4_small_kernel(Layer L, const __half* __restrict__ X, int M, int64_t ldx,
                                                             __half* __restrict__ Y, int64_t ldy, SmallLds ld, int KS, int ks_magic,
                                                             GroupTail G, const int* __restrict__ perm) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // no integer division here: the launch is short enough for its emulation to show (TW <= 4;
    // a / KS = a * ks_magic >> 16 with ks_magic = ceil(65536 / KS), exact for a < 4096)
    const int ti = (wave >= KS) + (wave >= 2 * KS) + (wave >= 3 * KS), kw = wave - ti * KS;  // tile within the workgroup, K split index
    const int TW = ld.tw;
    const int n = lane & 15, kb = lane >> 4;
    // which layer of the group this wave's tile belongs to (a workgroup may straddle two)
    int tile = blockIdx.x * TW + ti;
    const int li = (tile >= G.tile_begin[0]) + (tile >= G.tile_begin[1]) + (tile >= G.tile_begin[2]);
    if (li > 0) {
        L.qweight = G.qweight[li - 1];
        L.scales = G.scales[li - 1];
        L.zeros = G.zeros[li - 1];
        L.weak = G.weak[li - 1];
        L.oc = G.oc[li - 1];
        Y = G.Y[li - 1];
        ldy = G.ldy[li - 1];
        tile -= G.tile_begin[li - 1];
    }
    const int row0 = tile * 16;
    const int nq = L.ng;
    const int units = (nq + 3) >> 2;
    const int q_beg = 4 * ((units * kw * ks_magic) >> 16);
    const int q_end = min(4 * ((units * (kw + 1) * ks_magic) >> 16), nq);
    const int nj = max(q_end - q_beg, 0);
    const int nweak = (L.k + 31) / 32;
    const u4 zero4 = u4{0u, 0u, 0u, 0u};
    const bool has_x = n < M;

    // ---- requests -------------------------------------------------------------------------------------
    const int orow = min(row0 + n, L.oc - 1);
    const int per_m = nq * 16;
    const int total = M * per_m;  // X fragments: idx -> (row m, fragment f of 8 columns); multiple of 16
    u4 xv[4];
    int xm[4], xf[4];
    // 8 activations of row m at stored columns c0 .. c0 + 7 (c0 a multiple of 8)
    auto table8 = [&](int c0, u4& lo, u4& hi) {
        lo = load16(perm + c0);
        hi = load16(perm + c0 + 4);
    };
    auto gather8 = [&](int m, u4 lo, u4 hi) {
        const unsigned short* row = reinterpret_cast<const unsigned short*>(X) + (size_t)m * ldx;
        uint32_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = row[min(max((int)(e < 4 ? lo[e] : hi[e - 4]), 0), L.ic - 1)];
        return u4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
    };
    u4 tlo[4], thi[4];
    int xrow[4];
    auto load_x = [&](int base) {   // with a table: its entries only; gather_x() then fetches the activations
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = base + u * blockDim.x + threadIdx.x;
            const int cidx = min(idx, total - 1);
            const int m = (cidx >= per_m) + (cidx >= 2 * per_m) + (cidx >= 3 * per_m);
            xm[u] = (idx < total) ? m : -1;
            xrow[u] = m;
            xf[u] = cidx - m * per_m;
            // fragments past Kq (the last group's padding) read the row's last quantized fragment and are zeroed below
            if (PERM) table8(min(8 * xf[u], L.kq - 8), tlo[u], thi[u]);
            else xv[u] = load16(X + (size_t)m * ldx + min(8 * xf[u], L.kq - 8));
        }
    };
    auto gather_x = [&]() {
        if (PERM) {
#pragma unroll
            for (int u = 0; u < 4; ++u) xv[u] = gather8(xrow[u], tlo[u], thi[u]);
        }
    };
    auto store_x = [&]() {   // Sx of a group lands with its first fragment
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (8 * xf[u] >= L.kq) xv[u] = zero4;
            const float t = sum16(sum8(xv[u]));
            if (xm[u] >= 0) {
                *reinterpret_cast<u4*>(lds + xm[u] * ld.xrow + xf[u] * 16) = W3 ? xv[u] : permute_x(xv[u]);
                if ((xf[u] & 15) == 0) reinterpret_cast<float*>(lds + ld.sx_off)[(xf[u] >> 4) * 4 + xm[u]] = t;
            }
        }
    };
    load_x(0);
    // group parameters of this wave's tile: chunk c = array c % 2 (scales, zero-points), groups
    // 32 (c / 2) + 8 kb .. + 7 of row n; chunks kw, kw + KS, ... (a chunk past the end repeats the last)
    const int nchunks = 2 * ((nq + 31) >> 5);
    u4 pv[NSZ];
#pragma unroll
    for (int i = 0; i < NSZ; ++i) {
        const int c = min(kw + i * KS, nchunks - 1);
        const int g0 = min(32 * (c >> 1) + 8 * kb, (int)L.gs - 8);
        pv[i] = load16(((c & 1) ? L.zeros : L.scales) + (size_t)orow * L.gs + g0);
    }
    // weights: steps past the wave's range re-read its last step (never consumed)
    constexpr int WSTEP = W3 ? 48 : 64, WLANE = W3 ? 12 : 16;   // bytes of a row per step, and per lane
    const unsigned char* wp =
        reinterpret_cast<const unsigned char*>(L.qweight + (size_t)orow * L.stride) + WSTEP * (size_t)q_beg + WLANE * kb;
    auto load_w = [&](const unsigned char* p) {
        if (W3) {
            const uint32_t* q = reinterpret_cast<const uint32_t*>(p);
            return u4{q[0], q[1], q[2], 0u};
        }
        return load16(p);
    };
    const int j_last = max(min(nj, nq - q_beg) - 1, 0);
    u4 wq[D];
#pragma unroll
    for (int d = 0; d < D; ++d) wq[d] = load_w(wp + WSTEP * min(d, j_last));
    // weak steps of 32 fp16 columns are dealt to the K-split waves from the last one back
    // (columns past k are clamped here and zeroed where they are used; k >= 8)
    u4 wk[WMAX], xw[WMAX], wlo[WMAX], whi[WMAX];
    const int mrow = min(n, M - 1);
#pragma unroll
    for (int i = 0; i < WMAX; ++i) {
        const int c0 = min(32 * (KS - 1 - kw + i * KS) + 8 * kb, L.k - 8);
        wk[i] = load16(L.weak + (size_t)orow * L.k + c0);
        if (PERM) table8(L.kq + c0, wlo[i], whi[i]);
        else xw[i] = load16(X + (size_t)mrow * ldx + L.kq + c0);
    }
    __builtin_amdgcn_sched_barrier(0);   // nothing below may move above the requests
    if (PERM) {   // the table entries were requested first and arrive first: now the activations themselves
        gather_x();
#pragma unroll
        for (int i = 0; i < WMAX; ++i) xw[i] = gather8(mrow, wlo[i], whi[i]);
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- stage X (permuted, with Sx) and the group parameters ----------------------------------------
    store_x();
    {
        float* szt = reinterpret_cast<float*>(lds + ld.sz_off + (size_t)ti * ld.sz_tile);
#pragma unroll
        for (int i = 0; i < NSZ; ++i) {
            const int c = kw + i * KS;
            const int g0 = 32 * (c >> 1) + 8 * kb;
            const h8 h = as_h8(pv[i]);
            if (c < nchunks) {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (g0 + e < nq) szt[((g0 + e) * 16 + n) * 2 + (c & 1)] = (c & 1) ? 1024.f + (float)h[e] : (float)h[e];
            }
        }
    }
    for (int base = 4 * blockDim.x; base < total; base += 4 * blockDim.x) {   // only when X exceeds one pass
        load_x(base);
        gather_x();
        store_x();
    }
    // rows of Sx beyond M read as zero
    for (int i = threadIdx.x; i < nq * 4; i += blockDim.x)
        if ((i & 3) >= M) reinterpret_cast<float*>(lds + ld.sx_off)[i] = 0.f;
    for (int i = threadIdx.x; i < 64 * 8; i += blockDim.x) reinterpret_cast<float*>(lds + ld.zero_off)[i] = 0.f;
    __syncthreads();

    // ---- stream this wave's steps ---------------------------------------------------------------------
    f4 y[1];
    y[0] = f4{0.f, 0.f, 0.f, 0.f};
    const Consts magic = make_consts(W3 ? 0x00070007u : 0x000f000fu);
    // lanes without an activation row (n >= M), and accumulator rows >= 4 for Sx, read zero bytes
    const bool has_sx = kb == 0;
    int xa_addr = has_x ? n * ld.xrow + kb * 64 + q_beg * 256 : ld.zero_off;
    int sx_addr = has_sx ? ld.sx_off + q_beg * 16 : ld.zero_off;
    int sz_addr = ld.sz_off + ti * ld.sz_tile + q_beg * 128 + n * 8;
    const int xa_inc = has_x ? 256 * D : 0, sx_inc = has_sx ? 16 * D : 0;

    auto step = [&](int d) {
        u4 xa[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) xa[i] = *reinterpret_cast<const u4*>(lds + xa_addr + d * 256 + 16 * i);
        const f4 sx = *reinterpret_cast<const f4*>(lds + sx_addr + d * 16);
        const float2 sz = *reinterpret_cast<const float2*>(lds + sz_addr + d * 128);
        step_tile<W3>(y[0], xa, wq[d], sx, sz.x, sz.y, magic);
    };
    auto advance = [&]() {
        wp += WSTEP * D;
        xa_addr += xa_inc;
        sx_addr += sx_inc;
        sz_addr += 128 * D;
    };

    int j0 = 0;
    for (; j0 + 2 * D <= nj; j0 += D) {  // steady state: every load is real, no branches
#pragma unroll
        for (int d = 0; d < D; ++d) {
            step(d);
            wq[d] = load_w(wp + WSTEP * (d + D));
            __builtin_amdgcn_sched_barrier(0);  // keep the refill right behind its step: D loads stay in flight
        }
        advance();
    }
    for (; j0 < nj; j0 += D) {  // last < 2*D steps
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (j0 + d < nj) {
                step(d);
                if (j0 + d + D < nj) wq[d] = load_w(wp + WSTEP * (d + D));
            }
        }
        advance();
    }
    // ---- weak block ---------------------------------------------------------------------------------------
#pragma unroll
    for (int i = 0; i < WMAX; ++i)
        if (KS - 1 - kw + i * KS < nweak) {
            const bool live = has_x && 32 * (KS - 1 - kw + i * KS) + 8 * kb < L.k;
            y[0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(live ? xw[i] : zero4), as_h8(wk[i]), y[0], 0, 0, 0);
        }
    reduce_store<1>(L, y, kw, KS, lane, row0, M, Y, ldy, [&](int w) {
        return reinterpret_cast<float*>(lds + ld.red_off) + (size_t)(ti * (KS - 1) + (w - 1)) * 4 * 64;
    });
}

// =============================================================================================
// Chunked kernel: any M <= 16, R tiles per wave share the A fragments; each wave stages CH steps
// of its own K range at a time into a private LDS region.
// =============================================================================================
constexpr int XROW = 272;  // bytes per activation row and step: 16 fragments + 16 B against bank conflicts

template <int R, int CH>
struct Region {
    int xstep;  // bytes of X per step
    __device__ __forceinline__ Region(int M) : xstep(M * XROW) {}
    __device__ __forceinline__ int x_off(int sl) const { return sl * xstep; }
    __device__ __forceinline__ int sx_off(int sl) const { return CH * xstep + sl * 64; }
    __device__ __forceinline__ int s_off(int sl) const { return CH * xstep + CH * 64 + sl * (R * 64); }
    __device__ __forceinline__ int z_off(int sl) const { return CH * xstep + CH * 64 + CH * R * 64 + sl * (R * 64); }
};
inline size_t region_bytes(int R, int CH, int M) {
    const size_t b = (size_t)CH * ((size_t)M * XROW + 64 + 2 * (size_t)R * 64);
    const size_t red = (size_t)R * 4 * 64 * sizeof(float);  // the region doubles as the reduction buffer
    return b > red ? b : red;
}

// R: row tiles per wave, D: weight loads in flight per tile, CH: steps staged per chunk (multiple of D)
template <int R, int D, int CH>
__global__ __launch_bounds__(512) void gemv_w4_chunk_kernel(Layer L, const __half* __restrict__ X, int M, int64_t ldx,
                                                            __half* __restrict__ Y, int64_t ldy, int region_stride) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int lane = threadIdx.x & 63;
    const int KS = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, kb = lane >> 4;
    const int row0 = blockIdx.x * (16 * R);
    unsigned char* my = lds + (size_t)wave * region_stride;
    const Region<R, CH> rg(M);

    const int nq = L.ng;
    const int q_beg = (int)((int64_t)nq * wave / KS), q_end = (int)((int64_t)nq * (wave + 1) / KS);
    const int nj = q_end - q_beg;

    const unsigned char* wrow[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int o = min(row0 + 16 * r + n, L.oc - 1);
        wrow[r] = reinterpret_cast<const unsigned char*>(L.qweight + (size_t)o * L.stride) + 64 * (size_t)q_beg + 16 * kb;
    }
    const bool mvalid = n < M;
    const Consts magic = make_consts();

    f4 y[R];
#pragma unroll
    for (int r = 0; r < R; ++r) y[r] = f4{0.f, 0.f, 0.f, 0.f};
    const u4 zero4 = u4{0u, 0u, 0u, 0u};

    u4 wq[D][R];
    auto load_w = [&](int d, int j) {  // j: step index local to this wave
#pragma unroll
        for (int r = 0; r < R; ++r) wq[d][r] = load16(wrow[r] + 64 * (size_t)j);
    };
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (d < nj) load_w(d, d);

    // rows of Sx that no activation row fills stay zero
    for (int i = lane; i < CH * 16; i += 64) reinterpret_cast<float*>(my + rg.sx_off(0))[i] = 0.f;

    for (int c0 = 0; c0 < nj; c0 += CH) {
        const int cs = min(CH, nj - c0);
        wave_lds_fence();
        // ---- stage X (permuted), Sx, scales and zero-points of steps [c0, c0+cs) -------------
        {
            const int per_m = cs * 16;    // fragments per activation row
            const int total = M * per_m;  // multiple of 16: a 16-lane group is all in or all out
            for (int base = 0; base < total; base += 64) {
                const int idx = base + lane;
                const bool in = idx < total;
                const int m = in ? idx / per_m : 0;
                const int jj = in ? idx % per_m : 0;
                const int sl = jj >> 4, f = jj & 15;
                const int col = (q_beg + c0 + sl) * 128 + 8 * f;
                u4 v = zero4;
                if (in && col < L.kq) v = load16(X + (size_t)m * ldx + col);
                const float t = sum16(sum8(v));
                if (in) {
                    *reinterpret_cast<u4*>(my + rg.x_off(sl) + m * XROW + f * 16) = permute_x(v);
                    if (f == 0) reinterpret_cast<float*>(my + rg.sx_off(sl))[m] = t;
                }
            }
            const int totp = R * 16 * cs;
            for (int idx = lane; idx < totp; idx += 64) {
                const int sl = idx % cs, ri = idx / cs;
                const int o = min(row0 + ri, L.oc - 1);
                const size_t gi = (size_t)o * L.gs + q_beg + c0 + sl;
                reinterpret_cast<float*>(my + rg.s_off(sl))[ri] = __half2float(L.scales[gi]);
                reinterpret_cast<float*>(my + rg.z_off(sl))[ri] = 1024.f + __half2float(L.zeros[gi]);
            }
        }
        wave_lds_fence();
        // ---- stream the weights of the chunk -------------------------------------------------
        for (int sl0 = 0; sl0 < cs; sl0 += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const int sl = sl0 + d;
                if (sl < cs) {
                    u4 xa[4];
                    const unsigned char* xp = my + rg.x_off(sl) + n * XROW + kb * 64;
#pragma unroll
                    for (int i = 0; i < 4; ++i) xa[i] = mvalid ? *reinterpret_cast<const u4*>(xp + 16 * i) : zero4;
                    const f4 sx = *reinterpret_cast<const f4*>(my + rg.sx_off(sl) + kb * 16);
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        const float sf = reinterpret_cast<const float*>(my + rg.s_off(sl))[16 * r + n];
                        const float c = reinterpret_cast<const float*>(my + rg.z_off(sl))[16 * r + n];
                        step_tile(y[r], xa, wq[d][r], sx, sf, c, magic);
                    }
                    const int jn = c0 + sl + D;  // refill this slot with the step D ahead
                    if (jn < nj) load_w(d, jn);
                }
            }
        }
    }

    weak_steps<R>(L, X, M, ldx, row0, wave, KS, n, kb, y);
    wave_lds_fence();
    reduce_store<R>(L, y, wave, KS, lane, row0, M, Y, ldy,
                    [&](int w) { return reinterpret_cast<float*>(lds + (size_t)w * region_stride); });
}

template <int R, int D, int CH>
hipError_t launch_chunk(const Layer& L, const __half* X, int M, int64_t ldx, __half* Y, int64_t ldy, int ks,
                        hipStream_t s) {
    const int grid = ceil_div(L.oc, 16 * R);
    const size_t region = (region_bytes(R, CH, M) + 255) / 256 * 256;
    gemv_w4_chunk_kernel<R, D, CH><<<grid, 64 * ks, region * ks, s>>>(L, X, M, ldx, Y, ldy, (int)region);
    return hipGetLastError();
}

// =============================================================================================
// Row-batch kernel: any M <= 16 without staging.  With more than a few activation rows X no
// longer fits in LDS, and staging it in chunks puts a load latency in front of every chunk.  Here
// a wave reads the A fragments it needs straight from X (L2-resident: every wave of the launch
// reads the same few hundred KB), D steps ahead like the weights, and permutes them in registers:
// lane (n, kb) takes for fragment i the 16 bytes X[n][128 j + 32 kb + 8 i ..] - the columns of word
// 4 kb + i of the step, which is the word its weight load puts in component i.  R tiles of 16 rows share each fragment, so X adds 4 / R
// requests per weight request.  The group sums Sx come from the matrix core: one more MFMA per
// fragment against an all-ones B operand leaves sum_k x[m][k] in the accumulator layout the
// zero-point correction needs.  Lanes past M read row M - 1: they only feed rows of the 16 x 16
// result that are never stored.  LDS is used for the final reduction over the K split only.
// =============================================================================================
template <int R, int D>
__global__ __launch_bounds__(512) void gemv_w4_rows_kernel(Layer L, const __half* __restrict__ X, int M, int64_t ldx,
                                                           __half* __restrict__ Y, int64_t ldy, int ks_magic) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int lane = threadIdx.x & 63;
    const int KS = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, kb = lane >> 4;
    const int row0 = blockIdx.x * (16 * R);
    const int nq = L.ng;
    const int units = (nq + 3) >> 2;
    const int q_beg = 4 * ((units * wave * ks_magic) >> 16);                 // a / KS = a * ceil(65536 / KS) >> 16
    const int q_end = min(4 * ((units * (wave + 1) * ks_magic) >> 16), nq);
    const int nj = max(q_end - q_beg, 0);
    const int j_last = max(nj - 1, 0);
    const Consts magic = make_consts();
    u4 ones = u4{0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
    asm volatile("" : "+v"(ones.x), "+v"(ones.y), "+v"(ones.z), "+v"(ones.w));

    const unsigned char* wrow[R];
    const __half *sp[R], *zp[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int o = min(row0 + 16 * r + n, L.oc - 1);
        wrow[r] = reinterpret_cast<const unsigned char*>(L.qweight + (size_t)o * L.stride) + 64 * (size_t)q_beg + 16 * kb;
        sp[r] = L.scales + (size_t)o * L.gs + q_beg;
        zp[r] = L.zeros + (size_t)o * L.gs + q_beg;
    }
    // fragment i of step j: columns 128 (q_beg + j) + 32 kb + 8 i; the last group may be partial
    // (a fragment past Kq re-reads the row's last quantized fragment and is zeroed where it is used)
    const __half* xrow = X + (size_t)min(n, M - 1) * ldx;
    const int col0 = 128 * q_beg + 32 * kb;

    u4 xq[D][4], wq[D][R];
    u2 sb[D / 4 > 0 ? D / 4 : 1][R], zb[D / 4 > 0 ? D / 4 : 1][R];
    static_assert(D % 4 == 0, "scales are fetched four steps at a time");
    auto load_step = [&](int d, int j) {   // straight-line: the step index is clamped, never tested
        const int jc = min(j, j_last);
#pragma unroll
        for (int i = 0; i < 4; ++i) xq[d][i] = load16(xrow + min(col0 + 128 * jc + 8 * i, L.kq - 8));
#pragma unroll
        for (int r = 0; r < R; ++r) wq[d][r] = load16(wrow[r] + 64 * (size_t)jc);
    };
    auto load_sz = [&](int c, int j) {     // steps j .. j + 3 (j a multiple of 4)
        const int jc = min(j, j_last & ~3);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            sb[c][r] = load8(sp[r] + jc);
            zb[c][r] = load8(zp[r] + jc);
        }
    };
#pragma unroll
    for (int d = 0; d < D; ++d) {
        if ((d & 3) == 0) load_sz(d >> 2, d);
        load_step(d, d);
    }

    f4 y[R];
#pragma unroll
    for (int r = 0; r < R; ++r) y[r] = f4{0.f, 0.f, 0.f, 0.f};
    const u4 zero4 = u4{0u, 0u, 0u, 0u};

    auto step = [&](int d, int j) {
        u4 xa[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) xa[i] = permute_x((col0 + 128 * j + 8 * i < L.kq && j < nj) ? xq[d][i] : zero4);
        f4 sx = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 4; ++i) sx = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(xa[i]), as_h8(ones), sx, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float sf = half_at(sb[d >> 2][r], d & 3), c = 1024.f + half_at(zb[d >> 2][r], d & 3);
            step_tile(y[r], xa, wq[d][r], sx, sf, c, magic);
        }
    };

    // no branches inside: steps past the wave's range run on clamped loads and zeroed activations
    for (int j0 = 0; j0 < nj; j0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            step(d, j0 + d);
            load_step(d, j0 + d + D);
            if ((d & 3) == 3) load_sz(d >> 2, j0 + D + d - 3);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    weak_steps<R>(L, X, M, ldx, row0, wave, KS, n, kb, y);
    reduce_store<R>(L, y, wave, KS, lane, row0, M, Y, ldy,
                    [&](int w) { return reinterpret_cast<float*>(lds) + (size_t)(w - 1) * R * 4 * 64; });
}

template <int R, int D>
hipError_t launch_rows(const Layer& L, const __half* X, int M, int64_t ldx, __half* Y, int64_t ldy, int ks, hipStream_t s) {
    const int grid = ceil_div(L.oc, 16 * R);
    const size_t lds_bytes = (size_t)(ks > 1 ? ks - 1 : 1) * R * 4 * 64 * sizeof(float);
    gemv_w4_rows_kernel<R, D><<<grid, 64 * ks, lds_bytes, s>>>(L, X, M, ldx, Y, ldy, ceil_div(65536, ks));
    return hipGetLastError();
}

// =============================================================================================
// 3-bit kernel: any M <= 16.  Ten codes fill a 32-bit word, so a lane's 128-bit load holds 40
// consecutive codes of its row and a step of the four k-slot lanes covers 160 columns - groups
// of 128 columns do not line up with anything the matrix core sums over.  Dequantization is
// therefore done on the weight side: the 40 codes become five B fragments of 8 fp16 weights
// (q - z) s each, and five 16x16x32 MFMAs per step accumulate straight into the result.
//   * a word holds exactly five pairs of codes, so a pair never straddles words: its two codes are
//     spread to bits 0..2 and 16..18 by one 6-bit field extract and one multiplication by
//     2^13 + 1, then masked and or-ed with the exponent bits (3 instructions per 2 codes);
//   * fragment s of lane (n, kb) covers columns 160 j + 40 kb + 8 s .. + 7: one group, since
//     every such octet starts on a multiple of 8; its (zero-point, scale) pair comes from a table
//     of the tile's rows in LDS, filled once per workgroup with the same 16-byte-per-lane loads
//     of 8 groups as in the 4-bit kernel;
//   * activations are read from X as they are (natural column order), D steps ahead like the
//     weights, and shared by the R tiles of a wave; octets past Kq are zeroed.
// LDS: (z, s) fp16 pairs [groups][16 R rows] | reduction slots
// =============================================================================================
// DENSE: the dense 3-bit layout (a row is one bit string, 32 codes in 3 words).  A lane then takes
// 12 bytes = 32 codes = four fragments per step, a step of the four k-slot lanes covers exactly one group
// of 128 columns, and pair P of a lane sits at bits 6 P of its 96: two of the sixteen pairs straddle words
// and take one funnel shift more.  Group = step is what lets the dequantization move to the accumulator
// side (see step_dense): about half the vector instructions of the whole-codes-per-word layout.
template <int R, int D, int NSZ, bool DENSE>
__global__ __launch_bounds__(512) void gemv_w3_kernel(Layer L, const __half* __restrict__ X, int M, int64_t ldx,
                                                      __half* __restrict__ Y, int64_t ldy, int ks_magic, int nsteps) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int lane = threadIdx.x & 63;
    const int KS = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, kb = lane >> 4;
    const int row0 = blockIdx.x * (16 * R);
    const int q_beg = (nsteps * wave * ks_magic) >> 16;                 // a / KS = a * ceil(65536 / KS) >> 16
    const int q_end = (nsteps * (wave + 1) * ks_magic) >> 16;
    const int nj = max(q_end - q_beg, 0);
    const int j_last = max(nj - 1, 0);
    const int nq = L.ng;

    // ---- requests: group parameters of the workgroup's rows first, then D steps of X and weights ----
    // chunk c = (tile c / (2 nch), array c % 2, groups 32 (c / 2 % nch) ..): 8 groups per lane
    const int nch = (nq + 31) >> 5, nchunks = 2 * nch * R;
    u4 pv[NSZ];
#pragma unroll
    for (int i = 0; i < NSZ; ++i) {
        const int c = min(wave + i * KS, nchunks - 1);
        const int r = c / (2 * nch), cc = c - r * 2 * nch;
        const int o = min(row0 + 16 * r + n, L.oc - 1);
        const int g0 = min(32 * (cc >> 1) + 8 * kb, (int)L.gs - 8);
        pv[i] = load16(((cc & 1) ? L.zeros : L.scales) + (size_t)o * L.gs + g0);
    }
    constexpr int NF = DENSE ? 4 : 5;                 // fragments (octets of columns) per lane and step
    constexpr int STEP_COLS = 32 * NF, LANE_COLS = 8 * NF;
    constexpr int STEP_BYTES = DENSE ? 48 : 64, LANE_BYTES = DENSE ? 12 : 16;
    const unsigned char* wrow[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int o = min(row0 + 16 * r + n, L.oc - 1);
        wrow[r] = reinterpret_cast<const unsigned char*>(L.qweight + (size_t)o * L.stride);
    }
    const int woff0 = STEP_BYTES * q_beg + LANE_BYTES * kb;
    const int woff_max = 4 * L.stride - LANE_BYTES;   // never reached: the host admits only rows that hold whole steps
    const __half* xrow = X + (size_t)min(n, M - 1) * ldx;
    const int col0 = STEP_COLS * q_beg + LANE_COLS * kb;
    u4 xq[D][NF], wq[D][R];
    auto load_step = [&](int d, int j) {   // straight-line: the step index is clamped, never tested
        const int jc = min(j, j_last);
#pragma unroll
        for (int s = 0; s < NF; ++s) xq[d][s] = load16(xrow + min(col0 + STEP_COLS * jc + 8 * s, L.kq - 8));
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (DENSE) {
                const uint32_t* p = reinterpret_cast<const uint32_t*>(wrow[r] + min(woff0 + STEP_BYTES * jc, woff_max));
                wq[d][r] = u4{p[0], p[1], p[2], 0u};
            } else {
                wq[d][r] = load16(wrow[r] + woff0 + STEP_BYTES * (size_t)jc);
            }
        }
    };
#pragma unroll
    for (int d = 0; d < D; ++d) load_step(d, d);
    __builtin_amdgcn_sched_barrier(0);   // nothing below may move above the requests

    // ---- the (zero-point, scale) table ---------------------------------------------------------------
    unsigned short* szt = reinterpret_cast<unsigned short*>(lds);   // [group][16 R rows][z, s]
#pragma unroll
    for (int i = 0; i < NSZ; ++i) {
        const int c = wave + i * KS;
        const int r = c / (2 * nch), cc = c - r * 2 * nch;
        const int g0 = 32 * (cc >> 1) + 8 * kb;
        if (c < nchunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (g0 + e < nq) szt[((g0 + e) * (16 * R) + 16 * r + n) * 2 + ((cc & 1) ? 0 : 1)] = (unsigned short)(pv[i][e >> 1] >> (16 * (e & 1)));
        }
    }
    __syncthreads();

    f4 y[R];
#pragma unroll
    for (int r = 0; r < R; ++r) y[r] = f4{0.f, 0.f, 0.f, 0.f};
    const u4 zero4 = u4{0u, 0u, 0u, 0u};
    uint32_t cmask = 0x00070007u, cmagic = 0x64006400u;
    asm volatile("" : "+v"(cmask), "+v"(cmagic));
    const h2 k1024 = h2{(_Float16)1024.f, (_Float16)1024.f};
    const uint32_t* sz32 = reinterpret_cast<const uint32_t*>(lds);

    // a lane's 40 columns of a step touch at most two groups: both (zero-point, scale) pairs are read
    // one step ahead, and each fragment picks its own by comparing its first column with the boundary
    uint32_t zs_lo[R], zs_hi[R];
    const uint32_t* szl = sz32 + n;
    auto read_zs = [&](int j) {
        const int g = min((col0 + STEP_COLS * j) >> 7, nq - 1), gh = min(g + 1, nq - 1);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            zs_lo[r] = szl[g * (16 * R) + 16 * r];
            zs_hi[r] = szl[gh * (16 * R) + 16 * r];
        }
    };
    read_zs(0);
    u4 ones = u4{0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
    asm volatile("" : "+v"(ones.x), "+v"(ones.y), "+v"(ones.z), "+v"(ones.w));
    // Dense layout: a step is one group, so the dequantization moves behind the matrix cores as in the
    // 4-bit kernels: the codes enter as the exact fp16 numbers 1024 + q (three instructions per pair), the
    // step's sum over its 128 columns is taken in a fresh accumulator, and the group contributes
    // s (sum x (1024 + q) - (1024 + z) sum x); sum x comes from four more MFMAs against an all-ones
    // operand, shared by the R tiles, and lands in the accumulator's own layout.
    auto step_dense = [&](int d, int j) {
        const int col = col0 + STEP_COLS * j;
        float sc[R], tc[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const h2 zs = __builtin_bit_cast(h2, zs_lo[r]);
            sc[r] = (float)zs.y;
            tc[r] = sc[r] * (1024.f + (float)zs.x);
        }
        read_zs(j + 1);
        f4 sx = f4{0.f, 0.f, 0.f, 0.f}, ya[R];
#pragma unroll
        for (int r = 0; r < R; ++r) ya[r] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < NF; ++s) {
            const u4 xa = (col + 8 * s < L.kq && j < nj) ? xq[d][s] : zero4;
            sx = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(xa), as_h8(ones), sx, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                u4 b;
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const int P = 4 * s + p;   // pair P of the lane's 16 at bits 6 P .. 6 P + 5 of its three words
                    const int wi = (6 * P) >> 5, sh = (6 * P) & 31;
                    const uint32_t six = sh <= 26 ? __builtin_amdgcn_ubfe(wq[d][r][wi], sh, 6)
                                                  : __builtin_amdgcn_ubfe(__builtin_amdgcn_alignbit(wq[d][r][(wi + 1) & 3], wq[d][r][wi], sh), 0, 6);
                    b[p] = ((six * 0x2001u) & cmask) | cmagic;   // fp16 pair (1024 + q0, 1024 + q1)
                }
                ya[r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(xa), as_h8(b), ya[r], 0, 0, 0);
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < 4; ++e) y[r][e] += sc[r] * ya[r][e] - tc[r] * sx[e];
    };
    auto step = [&](int d, int j) {
        if (DENSE) {
            step_dense(d, j);
            return;
        }
        const int col = col0 + STEP_COLS * j;
        const int split = ((col >> 7) + 1) << 7;   // first column of the next group
        h2 zsl[R], zsh[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            zsl[r] = __builtin_bit_cast(h2, zs_lo[r]);
            zsh[r] = __builtin_bit_cast(h2, zs_hi[r]);
        }
        read_zs(j + 1);
        f4 ya[R], yb[R];   // two accumulation chains per tile: consecutive MFMAs do not wait for each other
#pragma unroll
        for (int r = 0; r < R; ++r) ya[r] = yb[r] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < NF; ++s) {
            const u4 xa = (col + 8 * s < L.kq && j < nj) ? xq[d][s] : zero4;
            const bool hi = col + 8 * s >= split;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const h2 zs = hi ? zsh[r] : zsl[r];
                const h2 z2 = h2{zs.x, zs.x}, s2 = h2{zs.y, zs.y};
                u4 b;
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const int P = 4 * s + p;   // pair P of the lane's 20: word P / 5, codes 2 (P % 5) and the next
                    const uint32_t six = __builtin_amdgcn_ubfe(wq[d][r][P / 5], 6 * (P % 5), 6);
                    const uint32_t codes = ((six * 0x2001u) & cmask) | cmagic;   // fp16 pair (1024 + q0, 1024 + q1)
                    b[p] = __builtin_bit_cast(uint32_t, ((__builtin_bit_cast(h2, codes) - k1024) - z2) * s2);
                }
                if (s & 1) yb[r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(xa), as_h8(b), yb[r], 0, 0, 0);
                else ya[r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(xa), as_h8(b), ya[r], 0, 0, 0);
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < 4; ++e) y[r][e] += ya[r][e] + yb[r][e];
    };

    // no branches inside: steps past the wave's range run on clamped loads and zeroed activations
    for (int j0 = 0; j0 < nj; j0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            step(d, j0 + d);
            load_step(d, j0 + d + D);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    weak_steps<R>(L, X, M, ldx, row0, wave, KS, n, kb, y);
    __syncthreads();   // the table is dead: its memory becomes the reduction slots
    reduce_store<R>(L, y, wave, KS, lane, row0, M, Y, ldy,
                    [&](int w) { return reinterpret_cast<float*>(lds) + (size_t)(w - 1) * R * 4 * 64; });
}

// K-split waves of the 3-bit kernel: four (one per SIMD; measured best for 4096 ... 11008 rows), more only
// when the (zero-point, scale) table would otherwise take more than 4 requests per wave
int w3_steps(const Layer& L) { return L.dense ? L.ng : ceil_div(L.words, 16); }   // dense: one step per group

int w3_split(const Layer& L, int R) {
    const int nsteps = w3_steps(L), nchunks = 2 * ceil_div(L.ng, 32) * R;
    int ks = nsteps < 4 ? (nsteps < 1 ? 1 : nsteps) : 4;
    while (ks < 8 && ks < nsteps && ceil_div(nchunks, ks) > 4) ++ks;
    return ks;
}

template <int R>
hipError_t launch_w3(const Layer& L, const __half* X, int M, int64_t ldx, __half* Y, int64_t ldy, hipStream_t s) {
    const int tiles = ceil_div(L.oc, 16 * R);
    const int nsteps = w3_steps(L);
    const int ks = w3_split(L, R);
    const int nchunks = 2 * ceil_div(L.ng, 32) * R;
    const int nsz = ceil_div(nchunks, ks);
    const size_t table = (size_t)L.ng * 16 * R * 4, red = (size_t)(ks > 1 ? ks - 1 : 1) * R * 4 * 64 * sizeof(float);
    const size_t lds_bytes = table > red ? table : red;
    using Kern = void (*)(Layer, const __half*, int, int64_t, __half*, int64_t, int, int);
    static const Kern table_k[2][4] = {
        {gemv_w3_kernel<R, 4, 1, false>, gemv_w3_kernel<R, 4, 2, false>, gemv_w3_kernel<R, 4, 3, false>, gemv_w3_kernel<R, 4, 4, false>},
        {gemv_w3_kernel<R, 4, 1, true>, gemv_w3_kernel<R, 4, 2, true>, gemv_w3_kernel<R, 4, 3, true>, gemv_w3_kernel<R, 4, 4, true>}};
    if (nsz > 4 || lds_bytes > 64 * 1024) return hipErrorInvalidValue;   // not reached for the shapes gemv_supported admits
    table_k[L.dense ? 1 : 0][nsz - 1]<<<tiles, 64 * ks, lds_bytes, s>>>(L, X, M, ldx, Y, ldy, ceil_div(65536, ks), nsteps);
    return hipGetLastError();
}

// =============================================================================================
// Register kernel: 3 <= M <= 16, rows of any length in passes of (waves x S) steps.  A workgroup has one wave per K
// range of S steps, and lane (n, kb) of a wave keeps, for a whole pass, the A fragments of activation row n for its
// range (4 S registers of 8 halfs: the wave fetches its rows' 512 columns as whole kilobytes, deals them out through
// a private piece of LDS and permutes them once), together with the group sums Sx of its steps in accumulator layout
// (from MFMAs against an all-ones operand).  No workgroup-wide staging pass and no barrier before the stream: the
// weight requests go out with the first activation requests.  A workgroup walks T row tiles (compile-time, so every
// load is unconditional) with D tiles of weight loads in flight; the K-split partial tiles stay in registers
// and meet in LDS once, at the end.  Several layers that share X run as one launch (tiles of layer 0, 1, ...).
// =============================================================================================
struct RegsArgs {
    const uint32_t* qweight[MAX_GROUP];
    const __half* scales[MAX_GROUP];
    const __half* zeros[MAX_GROUP];
    const __half* weak[MAX_GROUP];
    __half* Y[MAX_GROUP];
    int64_t ldy[MAX_GROUP];
    int oc[MAX_GROUP];
    int tile_begin[MAX_GROUP];   // first 16-row tile of layer i; INT_MAX when absent
    int n_tiles;
    const __half* X;
    int64_t ldx;
    int M, kq, k, nq, stride, gs;
};

// S: steps per wave and pass; D: tiles in flight; T: tiles per workgroup; XM: activation rows fetched (8 or 16: one
// 128-bit load per row covers the wave's whole range - a contiguous kilobyte per request - and the fragments are
// dealt out through a wave-private piece of LDS; fetching every lane's fragments of its own row directly took 16
// requests of sixteen 64-byte pieces each and was 10 - 25 % slower on rows of more than one pass); MAXW: waves per
// workgroup at most (register budget); MULTI: rows longer than one pass of the workgroup (KS * S steps) take
// `passes` passes - the accumulators stay, the next pass's activation rows are requested as soon as this pass's
// sit in LDS, and the weight requests run on across the pass boundary (with several passes the tiles in flight
// must divide the tiles of a workgroup, because the slots are reused pass after pass: three tiles keep one in
// flight).  LDS: per wave max(XM, T) KB - first the activation bounce, at the end this wave's partial tiles.
template <int S, int D, int T, int XM, int MAXW, bool MULTI>
__global__ __launch_bounds__(64 * MAXW) void gemv_w4_regs_kernel(RegsArgs A, int passes) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    static_assert(S == 4, "a wave's range is 4 steps = 512 columns = 64 pieces of 16 bytes");
    static_assert(D == 1 || T % D == 0 || !MULTI, "with several passes the slots are reused pass after pass");
    constexpr int WKB = XM > T ? XM : T;   // KB of LDS per wave
    const int lane = threadIdx.x & 63;
    const int KS = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, kb = lane >> 4;
    const int nweak = (A.k + 31) >> 5;
    const int wt = min(wave, nweak - 1);            // weak step of this wave (waves past the block repeat the last, with zero activations)
    const u4 zero4 = u4{0u, 0u, 0u, 0u};
    const int C = MULTI ? passes : 1;
    unsigned char* mine = lds + (size_t)wave * (WKB * 1024);

    // ---- per-tile pointers (wave-uniform) and requests --------------------------------------------------------
    u4 wq[D][S], wk[D];
    u2 sb[D], zb[D];
    auto issue = [&](int d, int t, int c) {   // t: tile of this workgroup (compile-time), clamped to the launch's last tile; c: pass
        int tile_g = min((int)blockIdx.x * T + t, A.n_tiles - 1);
        // (opaque: with several passes the compiler would otherwise keep every tile's row addresses in registers
        // across the pass loop - 8 registers per tile - and spill the accumulators instead)
        if (MULTI) asm volatile("" : "+s"(tile_g));
        const int li = (tile_g >= A.tile_begin[1]) + (tile_g >= A.tile_begin[2]) + (tile_g >= A.tile_begin[3]);
        const int row0 = (tile_g - A.tile_begin[li]) * 16;
        const size_t orow = (size_t)min(row0 + n, A.oc[li] - 1);
        const int js0 = (min(c, C - 1) * KS + wave) * S;
        const unsigned char* wp = reinterpret_cast<const unsigned char*>(A.qweight[li] + orow * A.stride) + 16 * kb;
#pragma unroll
        for (int j = 0; j < S; ++j) wq[d][j] = load16(wp + 64 * min(js0 + j, (A.stride >> 4) - 1));
        const int g0 = min(js0, A.gs - S);
        sb[d] = load8(A.scales[li] + orow * A.gs + g0);
        zb[d] = load8(A.zeros[li] + orow * A.gs + g0);
        wk[d] = load16(A.weak[li] + orow * A.k + min(32 * wt + 8 * kb, A.k - 8));
    };

    const __half* xrow = A.X + (size_t)min(n, A.M - 1) * A.ldx;
    u4 xw = load16(xrow + A.kq + min(32 * wt + 8 * kb, A.k - 8));
    u4 ones = u4{0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
    asm volatile("" : "+v"(ones.x), "+v"(ones.y), "+v"(ones.z), "+v"(ones.w));
    const Consts magic = make_consts();
    f4 acc[T];
#pragma unroll
    for (int t = 0; t < T; ++t) acc[t] = f4{0.f, 0.f, 0.f, 0.f};

    // The activation rows of a pass: lane l fetches piece l (8 columns) of the wave's 512 columns, for each of the XM rows.
    // The registers are free again once the pieces sit in LDS, so with up to 8 rows the next pass's rows are requested
    // right there, ahead of this pass's products (columns past Kq: clamped, zeroed when used).
    u4 xrows[XM];
    auto fetch_x = [&](int c) {
        const int js0 = (c * KS + wave) * S;
#pragma unroll
        for (int m = 0; m < XM; ++m) xrows[m] = load16(A.X + (size_t)min(m, A.M - 1) * A.ldx + min(128 * js0 + 8 * lane, A.kq - 8));
    };
    // requests: the activations of this wave's first range (L2 hits), then the first D tiles of weights
    fetch_x(0);
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (d < T) issue(d, d, 0);
    __builtin_amdgcn_sched_barrier(0);   // nothing below may move above the requests

    // (with 16 rows the 64 registers of a second set of rows cost more in spilled accumulators than the fetch ahead
    // saves - 25 to 30 % on every 13B / 70B shape - so those fetch at the start of each pass)
    constexpr bool PREFETCH = MULTI && XM <= 8;
    // One pass over the workgroup's tiles with this wave's K range of pass c.
    auto pass = [&](int c, auto first_c) {
        constexpr bool FIRST = decltype(first_c)::value;   // the launch's first pass (it alone multiplies the weak block)
        const int js0 = (c * KS + wave) * S;   // first step of this wave in this pass
        // ---- this wave's activations for the pass: nibble order, zeros past M / Kq, group sums ---------------------
        // piece l of row m sits at chunk l ^ m of the row's KB: the 16 rows a fragment read touches at one chunk index
        // then spread over the banks (rows m and m + 8 share a bank group: the native two passes of a 128-bit read)
        u4 xa[S][4];
        if (MULTI && !PREFETCH && !FIRST) fetch_x(c);
#pragma unroll
        for (int m = 0; m < XM; ++m) *reinterpret_cast<u4*>(mine + 1024 * m + 16 * (lane ^ m)) = xrows[m];
        wave_lds_fence();
        if (PREFETCH) fetch_x(c + 1);
        const int nn = min(n, XM - 1);
        const unsigned char* src = mine + 1024 * nn;
#pragma unroll
        for (int j = 0; j < S; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) xa[j][i] = *reinterpret_cast<const u4*>(src + 16 * ((4 * kb + 16 * j + i) ^ nn));
        wave_lds_fence();
        f4 sx[S];
#pragma unroll
        for (int j = 0; j < S; ++j) {
            sx[j] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool live = n < A.M && 128 * (js0 + j) + 32 * kb + 8 * i < A.kq;
                xa[j][i] = permute_x(live ? xa[j][i] : zero4);
                sx[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(xa[j][i]), as_h8(ones), sx[j], 0, 0, 0);
            }
        }
        const u4 xwc = (FIRST && n < A.M && wave < nweak && 32 * wave + 8 * kb < A.k) ? xw : zero4;

#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int d = t % D;
#pragma unroll
            for (int j = 0; j < S; ++j) {
                const float sf = half_at(sb[d], j), cz = 1024.f + half_at(zb[d], j);
                step_tile(acc[t], xa[j], wq[d][j], sx[j], sf, cz, magic);
            }
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(xwc), as_h8(wk[d]), acc[t], 0, 0, 0);
            if (t + D < T) issue(d, t + D, c);
            else if (MULTI) issue(d, t + D - T, c + 1);   // the next pass's first tiles (D divides T; after the last pass: repeats, never used)
            __builtin_amdgcn_sched_barrier(0);   // keep the refill right behind its tile
        }
    };
    pass(0, std::true_type{});
#pragma clang loop unroll(disable)
    for (int c = 1; c < C; ++c) pass(c, std::false_type{});

    // ---- K split: partial tiles meet in LDS, wave t sums and stores tile t -----------------------------------------
#pragma unroll
    for (int t = 0; t < T; ++t) *reinterpret_cast<f4*>(mine + 1024 * t + 16 * lane) = acc[t];
    __syncthreads();
    for (int t = wave; t < T; t += KS) {
        const int tile_g = (int)blockIdx.x * T + t;
        if (tile_g >= A.n_tiles) break;
        f4 y = f4{0.f, 0.f, 0.f, 0.f};
        for (int w = 0; w < KS; ++w) {
            const f4 p = *reinterpret_cast<const f4*>(lds + (size_t)w * (WKB * 1024) + 1024 * t + 16 * lane);
#pragma unroll
            for (int e = 0; e < 4; ++e) y[e] += p[e];
        }
        const int li = (tile_g >= A.tile_begin[1]) + (tile_g >= A.tile_begin[2]) + (tile_g >= A.tile_begin[3]);
        const int o = (tile_g - A.tile_begin[li]) * 16 + n;
        __half* Y = A.Y[li];
        const int64_t ldy = A.ldy[li];
        // accumulator element e of lane l is row 4 * (l / 16) + e, column l % 16 of the 16 x 16 tile
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int m = 4 * kb + e;
            if (m < A.M && o < A.oc[li]) Y[(size_t)m * ldy + o] = __float2half_rn(y[e]);
        }
    }
}

constexpr int SMALL_LDS_LIMIT = 144 * 1024;   // of the 160 KB a CU has

}  // namespace

// the 3-bit kernel: its (zero-point, scale) table must fit in LDS and be loadable in 4 requests per wave
static bool w3_fits(const Layer& L) {
    // dense layout: a lane reads 12 bytes per group of its row, so whole groups must fit the padded row
    // (always true when Kq is a multiple of 128: 12 words per group)
    if (L.dense && 12 * L.ng > L.stride) return false;
    for (int R = 1; R <= 2; ++R) {
        const int ks = w3_split(L, R);
        if (ceil_div(2 * ceil_div(L.ng, 32) * R, ks) > 4 || (size_t)L.ng * 16 * R * 4 > 64 * 1024) return false;
    }
    return true;
}

bool gemv_supported(const Layer& L, int64_t M, int64_t ldx) {
    (void)ldx;
    if (M < 1 || L.g != 128 || (L.kq % 8) != 0 || (L.k % 8) != 0) return false;
    if (L.bits == 3) return L.kq >= 8 && w3_fits(L);
    return L.bits == 4;
}

namespace {
// The small-M kernel over `tiles` 16-row tiles (of one layer, or of a group's layers back to
// back).  Returns false when the configuration does not fit it; nothing is launched then.
bool launch_small(const Layer& L, int tiles, const GroupTail& tail, const int* perm, const __half* X, int M, int64_t ldx, __half* Y,
                  int64_t ldy, hipStream_t s, hipError_t* err) {
    const int units = (L.ng + 3) / 4;
    const int nweak = (L.k + 31) / 32;
    // K split in units of 4 steps over the waves of a workgroup, one row tile per workgroup.  Measured over the
    // Llama-2 7B / 13B / 70B launches (1 - 3 layers each): four waves - one per SIMD - are the best or within 3 %
    // of it whenever there are more row tiles than CUs, whatever the number of tiles (768 ... 3584) or units
    // (8 ... 56); more waves per tile only pay when there is at most one tile per CU and the rows are long
    // (4096 x 11008: six waves of <= 4 units).  At M = 1 several tiles per workgroup were never faster.
    const int ks_max = units < 1 ? 1 : (units > 16 ? 16 : units);
    int ks = 4;
    if (tiles <= 256 && units > 16) ks = ceil_div(units, 4);
    ks = ks > ks_max ? ks_max : ks;
    while (ks > 1 && ceil_div(units, ks - 1) == ceil_div(units, ks)) --ks;   // no wave with less than the longest share
    // the per-wave shares of the weak block and of the group parameters must fit the kernel's registers
    while (ks < ks_max && (ceil_div(nweak, ks) > 4 || ceil_div(2 * ceil_div(L.ng, 32), ks) > 3)) ++ks;
    // Every workgroup stages all of X (2 M IC bytes against the 8 IC bytes of a tile's codes): from M = 2 on,
    // 2 or 4 tiles share a workgroup's copy where that leaves at least a workgroup per CU, spread evenly
    // (28672 x 8192, M = 4: 36 us against 45; 8192 x 8192: 13.3 against 15.1; 11008 rows: no gain, 344
    // workgroups on 256 CUs)
    const auto even = [](int wgs) { return 5 * wgs >= 4 * 256 * ceil_div(wgs, 256); };
    int tw = 1;
    if (M >= 2 && tiles >= 512 && even(ceil_div(tiles, 2))) tw = 2;
    if (M >= 3 && tiles >= 1024 && even(ceil_div(tiles, 4))) tw = 4;
    if (ks * tw > 16) tw = 1;
    if (tw == 1 && ks < 8 && ks_max >= 8 && small_lds(M, L.ng, tw, ks).total > 64 * 1024) ks = 8;   // two workgroups per CU at most: larger ones
    const SmallLds ld = small_lds(M, L.ng, tw, ks);
    const int wmax = ceil_div(nweak, ks), nsz = ceil_div(2 * ceil_div(L.ng, 32), ks);
    if (!(ld.total <= SMALL_LDS_LIMIT && wmax <= 4 && nsz <= 3)) return false;
    using Kern = void (*)(Layer, const __half*, int, int64_t, __half*, int64_t, SmallLds, int, int, GroupTail, const int*);
    // prefetch depth: all of a wave's steps when it has at most 4, else 8 steps per lane unless
    // the weak prefetch already takes the registers (a request past the range would only repeat
    // the last one, but it still occupies the CU's address path at launch)
#define QEFT_SMALL_ROW(P, D, W, T) {gemv_w4_small_kernel<D, W, 1, P, T>, gemv_w4_small_kernel<D, W, 2, P, T>, gemv_w4_small_kernel<D, W, 3, P, T>}
    static const Kern table[3][4][3] = {
        {QEFT_SMALL_ROW(false, 4, 1, false), QEFT_SMALL_ROW(false, 8, 1, false), QEFT_SMALL_ROW(false, 8, 2, false), QEFT_SMALL_ROW(false, 4, 4, false)},
        {QEFT_SMALL_ROW(true, 4, 1, false), QEFT_SMALL_ROW(true, 8, 1, false), QEFT_SMALL_ROW(true, 8, 2, false), QEFT_SMALL_ROW(true, 4, 4, false)},
        {QEFT_SMALL_ROW(false, 4, 1, true), QEFT_SMALL_ROW(false, 8, 1, true), QEFT_SMALL_ROW(false, 8, 2, true), QEFT_SMALL_ROW(false, 4, 4, true)}};
#undef QEFT_SMALL_ROW
    static bool attr_set[3][4][3] = {};
    const int nj_max = 4 * ceil_div(units, ks);
    const int wi = wmax <= 1 ? (nj_max <= 4 ? 0 : 1) : (wmax <= 2 ? 2 : 3), si = nsz - 1;
    if (L.dense && perm) return false;   // no gathering variant for 3-bit codes
    const int pi = L.dense ? 2 : (perm ? 1 : 0);
    const Kern kern = table[pi][wi][si];
    if (!attr_set[pi][wi][si]) {
        *err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMALL_LDS_LIMIT);
        if (*err != hipSuccess) return true;
        attr_set[pi][wi][si] = true;
    }
    kern<<<ceil_div(tiles, tw), 64 * ks * tw, ld.total, s>>>(L, X, M, ldx, Y, ldy, ld, ks, ceil_div(65536, ks), tail, perm);
    *err = hipGetLastError();
    return true;
}

// The register kernel over the 16-row tiles of n layers that share X.  Returns false (nothing launched) when the
// shape does not fit it: not 4-bit / group 128, or a weak block wider than 32 columns per wave of the workgroup.
bool launch_regs(const Layer* Ls, int n, const __half* X, int M, int64_t ldx, __half* const* Y, const int64_t* ldy, hipStream_t s,
                 hipError_t* err) {
    const Layer& L = Ls[0];
    if (L.bits != 4 || L.dense || L.g != 128 || L.kq < 8 || L.k < 8 || (L.kq % 8) != 0 || (L.k % 8) != 0 || M < 3 || M > 16) return false;   // (one and two rows: the rows-per-wave and the staged kernels)
    constexpr int S = 4;
    // passes over K and waves per workgroup: at most 8 waves (two per SIMD keep the whole register file), rows longer
    // than 8 x 4 steps in the fewest passes
    const int units = ceil_div(L.ng, S);
    const int passes = ceil_div(units, 8), ks = ceil_div(units, passes);
    if (ceil_div(L.k, 32) > ks) return false;
    // three and four rows: only rows of a single pass (7B block at M = 4: 42.1 us with this kernel on q/k/v, o and
    // gate/up against 46.0 us on the staged kernel throughout; rows of several passes are faster there: 11.7 against 13.1 us)
    if (M < 5 && passes > 1) return false;
    RegsArgs A = {};
    int tiles = 0;
    for (int i = 0; i < MAX_GROUP; ++i) {
        const Layer& Li = Ls[i < n ? i : 0];
        A.qweight[i] = Li.qweight;
        A.scales[i] = Li.scales;
        A.zeros[i] = Li.zeros;
        A.weak[i] = Li.weak;
        A.Y[i] = Y[i < n ? i : 0];
        A.ldy[i] = ldy[i < n ? i : 0];
        A.oc[i] = Li.oc;
        A.tile_begin[i] = i < n ? tiles : INT_MAX;
        if (i < n) tiles += ceil_div(Li.oc, 16);
    }
    A.n_tiles = tiles;
    A.X = X;
    A.ldx = ldx;
    A.M = M;
    A.kq = L.kq;
    A.k = L.k;
    A.nq = L.ng;
    A.stride = L.stride;
    A.gs = L.gs;
    // tiles per workgroup (they share the activation registers): the fewest for which all workgroups are resident at
    // once - the register use of each variant and the LDS of a workgroup set how many a CU holds.
    static const int T_CHOICES[6] = {1, 2, 3, 4, 6, 8};
    // activation rows come as whole kilobytes per row and wave (8 or 16 requests) and are dealt out through LDS
    const int xi = M <= 8 ? 0 : 1, xm = M <= 8 ? 8 : 16;
    int ti = 0;
    for (; ti < 5; ++ti) {
        const int T = T_CHOICES[ti];
        const int waves_cu = passes > 1 ? 8 : (T <= 6 ? 12 : 8);   // from the variants' register counts (132 .. 166: three waves per SIMD; 186 .. 256: two)
        const int by_lds = (160 * 1024) / (ks * (xm > T ? xm : T) * 1024);
        int per_cu = waves_cu / ks < by_lds ? waves_cu / ks : by_lds;
        per_cu = per_cu < 1 ? 1 : per_cu;
        if (ceil_div(tiles, T) <= 256 * per_cu) break;
    }
    const int T = T_CHOICES[ti];
    const int grid = ceil_div(tiles, T);
    const size_t lds_bytes = (size_t)ks * (xm > T ? xm : T) * 1024;
    using Kern = void (*)(RegsArgs, int);
#define QEFT_REGS_ROW(XM, MU) {gemv_w4_regs_kernel<S, 1, 1, XM, 8, MU>, gemv_w4_regs_kernel<S, 2, 2, XM, 8, MU>, gemv_w4_regs_kernel<S, MU ? 1 : 2, 3, XM, 8, MU>, \
                               gemv_w4_regs_kernel<S, 2, 4, XM, 8, MU>, gemv_w4_regs_kernel<S, 2, 6, XM, 8, MU>, gemv_w4_regs_kernel<S, 2, 8, XM, 8, MU>}
    static const Kern table[2][2][6] = {{QEFT_REGS_ROW(8, false), QEFT_REGS_ROW(16, false)}, {QEFT_REGS_ROW(8, true), QEFT_REGS_ROW(16, true)}};
#undef QEFT_REGS_ROW
    static bool attr_set[2][2][6] = {};
    const Kern kern = table[passes > 1 ? 1 : 0][xi][ti];
    if (lds_bytes > 64 * 1024 && !attr_set[passes > 1 ? 1 : 0][xi][ti]) {
        *err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
        if (*err != hipSuccess) return true;
        attr_set[passes > 1 ? 1 : 0][xi][ti] = true;
    }
    kern<<<grid, 64 * ks, lds_bytes, s>>>(A, passes);
    *err = hipGetLastError();
    return true;
}

GroupTail no_tail() {
    GroupTail t = {};
    for (int i = 0; i < MAX_GROUP - 1; ++i) t.tile_begin[i] = INT_MAX;
    return t;
}
}  // namespace

hipError_t gemv_fwd_group(const Layer* Ls, int n, const __half* X, int64_t M64, int64_t ldx, __half* const* Y,
                          const int64_t* ldy, hipStream_t s, bool* handled) {
    *handled = false;
    const Layer& L = Ls[0];
    if (n < 1 || n > MAX_GROUP || M64 > 16 || L.kq < 8 || L.k < 8) return hipSuccess;
    if (M64 == 1) {   // one activation row: rows per wave, activations in registers
        hipError_t e = gemv_dot_fwd(Ls, n, nullptr, X, Y, s, handled);
        if (e != hipSuccess || *handled) return e;
    }
    if (M64 > 2) {    // 5 .. 16 rows: the register kernel (the small-M kernel below stages at most 4 rows); 3 and 4: where it is faster
        hipError_t e = hipSuccess;
        *handled = launch_regs(Ls, n, X, (int)M64, ldx, Y, ldy, s, &e);
        if (*handled || M64 > 4) return e;
    }
    if (!(L.bits == 4 || L.dense)) return hipSuccess;   // ten 3-bit codes per word: per-layer calls
    GroupTail tail = no_tail();
    int tiles = ceil_div(L.oc, 16);
    for (int i = 1; i < n; ++i) {
        tail.qweight[i - 1] = Ls[i].qweight;
        tail.scales[i - 1] = Ls[i].scales;
        tail.zeros[i - 1] = Ls[i].zeros;
        tail.weak[i - 1] = Ls[i].weak;
        tail.Y[i - 1] = Y[i];
        tail.ldy[i - 1] = ldy[i];
        tail.oc[i - 1] = Ls[i].oc;
        tail.tile_begin[i - 1] = tiles;
        tiles += ceil_div(Ls[i].oc, 16);
    }
    hipError_t err = hipSuccess;
    *handled = launch_small(L, tiles, tail, nullptr, X, (int)M64, ldx, Y[0], ldy[0], s, &err);
    return err;
}

hipError_t gemv_fwd_perm(const Layer& L, const int* perm, const __half* X, int64_t M64, int64_t ldx, __half* Y, int64_t ldy,
                         hipStream_t s, bool* handled) {
    *handled = false;
    if (M64 > 4 || L.bits != 4 || L.kq < 8 || L.k < 8) return hipSuccess;
    if (M64 == 1) {
        hipError_t e = gemv_dot_fwd(&L, 1, perm, X, &Y, s, handled);
        if (e != hipSuccess || *handled) return e;
    }
    hipError_t err = hipSuccess;
    *handled = launch_small(L, ceil_div(L.oc, 16), no_tail(), perm, X, (int)M64, ldx, Y, ldy, s, &err);
    return err;
}

hipError_t gemv_fwd(const Layer& L, const __half* X, int64_t M64, int64_t ldx, __half* Y, int64_t ldy, hipStream_t s) {
    const int M = (int)M64;
    if (M > 2) {      // 5 .. 16 rows: activations in registers, any row length; 3 and 4 rows: short rows only
        hipError_t e = hipSuccess;
        if (launch_regs(&L, 1, X, M, ldx, &Y, &ldy, s, &e)) return e;
    }
    if (M == 1) {
        bool handled = false;
        hipError_t e = gemv_dot_fwd(&L, 1, nullptr, X, &Y, s, &handled);
        if (e != hipSuccess || handled) return e;
    }
    if (M <= 4 && L.kq >= 8 && L.k >= 8 && (L.bits == 4 || L.dense)) {   // (dense 3-bit: gemv_supported has checked that rows hold whole steps)
        hipError_t err = hipSuccess;
        if (launch_small(L, ceil_div(L.oc, 16), no_tail(), nullptr, X, M, ldx, Y, ldy, s, &err)) return err;
    }
    if (L.bits == 3) return M > 4 ? launch_w3<2>(L, X, M, ldx, Y, ldy, s) : launch_w3<1>(L, X, M, ldx, Y, ldy, s);
    const int steps = L.ng + (L.k + 31) / 32;
    if (L.kq >= 8) {
        // unstaged kernel: R tiles per wave share the activation fragments; four K-split waves per workgroup
        // (one per SIMD), and four tiles per wave once that still leaves every CU more than two waves
        // (measured at M = 8 and 16: 4096 ... 8192 rows are 30 - 50 % faster with R = 2, 11008 ... 28672 rows
        // 5 - 25 % faster with R = 4; KS = 4 first or within 3 % of first on every shape)
        const int units = (L.ng + 3) / 4;
        const int R = ceil_div(L.oc, 64) >= 160 ? 4 : 2;
        int ks = units < 4 ? units : 4;
        ks = ks < 1 ? 1 : ks;
        if (R == 4) return launch_rows<4, 4>(L, X, M, ldx, Y, ldy, ks, s);
        return launch_rows<2, 4>(L, X, M, ldx, Y, ldy, ks, s);
    }
    const int R = (M <= 4) ? 1 : (M <= 8 ? 2 : 4);
    const int tiles = ceil_div(L.oc, 16 * R);
    int ks = ceil_div(2048, tiles);
    ks = ks < 1 ? 1 : (ks > 8 ? 8 : ks);
    while (ks > 1 && steps / ks < 2) --ks;
    if (R == 1) {
        if (M == 1) return launch_chunk<1, 4, 16>(L, X, M, ldx, Y, ldy, ks, s);
        if (M == 2) return launch_chunk<1, 4, 8>(L, X, M, ldx, Y, ldy, ks, s);
        return launch_chunk<1, 4, 4>(L, X, M, ldx, Y, ldy, ks, s);
    }
    if (R == 2) return launch_chunk<2, 2, 4>(L, X, M, ldx, Y, ldy, ks > 6 ? 6 : ks, s);
    return launch_chunk<4, 2, 2>(L, X, M, ldx, Y, ldy, ks > 6 ? 6 : ks, s);
}

}  // namespace qeft
