// Decode at M = 1 (paper Sec. 3.2.1): Y = x . W^T for one activation row, every stored byte of the layer
// streamed once.  A matrix-vector product has no reuse of the weights, so this kernel is shaped by the memory
// system alone:
//
//   * a wavefront owns whole weight rows.  One 128-bit load per lane covers 1 KB of contiguous codes of a row
//     (2048 columns, lane l the 32 columns 32 l .. 32 l + 31: a quarter of one 128-column group), so every
//     request is a full, contiguous kilobyte of one DRAM page;
//   * the activations live in registers for the whole launch: lane l keeps the 32 values of each of its column
//     ranges (NL ranges per wave), already in the order the nibbles leave the conversion, together with their
//     sums.  They are staged once per workgroup through LDS (coalesced read, transposed so that the per-lane
//     reads are conflict-free); after that the row loop touches neither LDS nor a barrier;
//   * dequantization is on the accumulator side: nibble pairs become the exact fp16 numbers 1024 + q (bits 0..3
//     of each half) and 64 + q (bits 4..7, no shift needed: the exponent of 64 gives mantissa bit 4 the weight 1),
//     two-element dot products accumulate x (base + q) in fp32, and the group's scale and zero-point are applied
//     to the lane's partial sum: s ((sum x (base + q) - sum base x) - z sum x).  Nothing is rounded to fp16;
//   * rows are dealt to the wavefronts in equal contiguous runs (DEPTH rows in flight, B batches per wave), the
//     loads of the next batch are issued as each row of the current one is consumed; there are no conditional
//     loads anywhere (rows past the end are clamped and never stored);
//   * a row's 64 lane sums are added with data-parallel-primitive moves; the wave's results are stored together.
//   * K can be split over KS waves of a workgroup when a row is too long for one wave's registers (the 70B
//     down projection); their partial results meet in LDS once, at the end.
//   * several layers that read the same input (q / k / v, gate / up) run as one launch: their rows are
//     concatenated and each row looks up its layer with scalar compares.
#include <climits>
#include <cstdlib>
#include <type_traits>

#include "qeft_internal.h"

namespace qeft {
namespace {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef uint32_t u3 __attribute__((ext_vector_type(3)));

constexpr int DOT_THREADS = 512;   // 8 waves: two per SIMD
constexpr int DOT_WAVES = DOT_THREADS / 64;

struct DotLayers {   // up to MAX_GROUP layers that share the input
    const uint32_t* qweight[MAX_GROUP];
    const __half* scales[MAX_GROUP];
    const __half* zeros[MAX_GROUP];
    const __half* weak[MAX_GROUP];
    __half* Y[MAX_GROUP];
    int oc[MAX_GROUP];
    int set_begin[MAX_GROUP];   // first row set (a wave's run of rows) of layer i; INT_MAX when absent
    int n_sets;
};

// a.x * b.x + a.y * b.y + c with fp32 products and sums
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, a), __builtin_bit_cast(h2, b), c, false);
}

// sum over the 64 lanes, valid in lane 63
__device__ __forceinline__ float wave_sum_to_lane63(float t) {
    auto dpp = [](float v, auto ctrl, auto rmask) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), decltype(ctrl)::value,
                                                                     decltype(rmask)::value, 0xf, false));
    };
    t += dpp(t, std::integral_constant<int, 0xB1>{}, std::integral_constant<int, 0xf>{});    // quad_perm [1,0,3,2]
    t += dpp(t, std::integral_constant<int, 0x4E>{}, std::integral_constant<int, 0xf>{});    // quad_perm [2,3,0,1]
    t += dpp(t, std::integral_constant<int, 0x141>{}, std::integral_constant<int, 0xf>{});   // row_half_mirror
    t += dpp(t, std::integral_constant<int, 0x140>{}, std::integral_constant<int, 0xf>{});   // row_mirror: every lane holds its row's sum
    t += dpp(t, std::integral_constant<int, 0x142>{}, std::integral_constant<int, 0xa>{});   // row_bcast15 into rows 1 and 3
    t += dpp(t, std::integral_constant<int, 0x143>{}, std::integral_constant<int, 0xc>{});   // row_bcast31 into rows 2 and 3
    return t;
}

// NL: 1 KB ranges of a row per wave (2048 columns each); DEPTH: rows in flight; NKW: weak columns per lane, in units of
// two (DEPTH 1) or four (DEPTH 2); PERM: gather the activations through the table while staging.
// With two rows in flight the rows go in pairs that share their small requests: the weak block of a pair comes
// with one load (lanes 0 .. 31 hold row 0's columns, lanes 32 .. 63 row 1's), and when a pair has at most four
// (row, range) slots, lane 4 g + m takes the parameters of slot m, so one 2-byte load per array serves both rows.
// LDS: pair-ordered activations [KS * NL][4 pieces][64 lanes] 16 B | (sum base x, sum x) float2 [KS * NL][64] |
//      weak activations fp16 | K-split exchange float [8 waves][64]
// W3D: three-bit codes in the dense layout (a row is one bit string, code j at bits 3 j .. 3 j + 2).  A lane's 32 columns
// are then 96 bits = three whole words (12-byte requests, 768 bytes per range and wave), its pairs (x_2P, x_2P+1) lie at
// bits 6 P of them - so the activations stay in column order - and both codes of a pair become 1024 + q: one 6-bit field
// extract (pairs 5 and 10 straddle words: a funnel shift first), one multiplication by 2^13 + 1, one and-or.
template <int NL, int DEPTH, int NKW, bool PERM, bool W3D>
__global__ __launch_bounds__(DOT_THREADS) void gemv_w4_dot_kernel(DotLayers R, int kq, int k, int row_bytes, int gs,
                                                                   const __half* __restrict__ X, const int* __restrict__ perm, int ic,
                                                                   int B, int ks_log2) {
    static_assert(DEPTH == 1 || DEPTH == 2, "one row or a pair of rows in flight");
    constexpr bool PAIR = DEPTH == 2;          // one weak load per pair of rows (no K split in these variants)
    constexpr bool PAIRP = PAIR && NL <= 2;    // one parameter load per array and pair
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int KS = PAIR ? 1 : (1 << ks_log2);
    const int kpart = PAIR ? 0 : (wave & (KS - 1)), wset = PAIR ? wave : (wave >> ks_log2);
    const int nl_all = NL * KS;                       // 1 KB ranges of a row, all waves of a K split together
    const int rpw = DEPTH * B;
    const int li0 = kpart * NL;
    // the wave's row set lies in ONE layer (each layer's rows are cut into sets of rpw on their own), looked up once
    const int sidx_raw = blockIdx.x * (PAIR ? DOT_WAVES : (DOT_WAVES >> ks_log2)) + wset;
    const bool live = sidx_raw < R.n_sets;
    const int sidx = min(sidx_raw, R.n_sets - 1);
    const int li = (sidx >= R.set_begin[1]) + (sidx >= R.set_begin[2]) + (sidx >= R.set_begin[3]);
    const int row_first = (sidx - R.set_begin[li]) * rpw, n_rows = R.oc[li];
    const unsigned char* const wbase = reinterpret_cast<const unsigned char*>(R.qweight[li]);
    const unsigned char* const sbase = reinterpret_cast<const unsigned char*>(R.scales[li]);
    const unsigned char* const zbase = reinterpret_cast<const unsigned char*>(R.zeros[li]);
    const unsigned char* const kbase_p = reinterpret_cast<const unsigned char*>(R.weak[li]);
    __half* const yout = R.Y[li];

    // ---- per-lane offsets of the wave's loads within a row (clamped: lanes past the row read its last bytes, their x is 0)
    // Group parameters: the four lanes of a quad share a group, so after a quad sum only one of them needs (s, z).
    // Per row: lane 4 g + m takes range 4 j + m of parameter set j.  Per pair (PAIRP): lane 4 g + m takes slot m =
    // (row m / NL of the pair, range m % NL).
    constexpr int NP = PAIRP ? 1 : (NL + 3) / 4;
    const int qm = lane & 3;
    const int p_row = PAIRP ? (qm >= NL ? 1 : 0) : 0, p_rng = PAIRP ? (qm >= NL ? qm - NL : qm) : 0;   // this lane's slot of a pair
    int woff[NL], goff[NP];
#pragma unroll
    for (int i = 0; i < NL; ++i) woff[i] = W3D ? min(768 * (li0 + i) + 12 * lane, row_bytes - 12) : min(1024 * (li0 + i) + 16 * lane, row_bytes - 16);
#pragma unroll
    for (int j = 0; j < NP; ++j) goff[j] = 2 * min(16 * (li0 + (PAIRP ? min(p_rng, NL - 1) : 4 * j + qm)) + (lane >> 2), gs - 1);
    // weak columns: DEPTH 1: dword t of the lane = columns 2 (lane + 64 (t KS + kpart)), + 1; pairs: the 4 NKW columns from
    // 4 NKW (lane % 32) on, of row lane / 32 of the pair
    constexpr int WKN = PAIR ? 2 * NKW : NKW;   // dwords of weak block per lane and load
    int koff[PAIR ? 1 : NKW];
    if (PAIR) {
        koff[0] = min(8 * NKW * (lane & 31), 2 * k - 8 * NKW);
    } else {
#pragma unroll
        for (int t = 0; t < NKW; ++t) koff[t] = 4 * min(lane + 64 * (t * KS + kpart), (k >> 1) - 1);
    }

    u4 wq[DEPTH][NL];
    uint32_t sq[PAIRP ? 1 : DEPTH][NP], zq[PAIRP ? 1 : DEPTH][NP], wk[PAIR ? 1 : DEPTH][WKN];
    auto issue_w = [&](int d, int row_in) {   // the codes of one row
        const unsigned char* wrow = wbase + (size_t)min(row_in, n_rows - 1) * (size_t)row_bytes;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            if (W3D) {
                const u3 v = *reinterpret_cast<const u3*>(wrow + woff[i]);
                wq[d][i] = u4{v.x, v.y, v.z, 0u};
            } else {
                wq[d][i] = *reinterpret_cast<const u4*>(wrow + woff[i]);
            }
        }
    };
    auto issue_small = [&](int d, int row_in) {   // group parameters and weak block: of row d (DEPTH 1, or the per-row parameters of a pair) ...
        const size_t lr = (size_t)min(row_in, n_rows - 1);
        if (!PAIRP) {
#pragma unroll
            for (int j = 0; j < NP; ++j) {
                sq[d][j] = *reinterpret_cast<const unsigned short*>(sbase + lr * (size_t)(2 * gs) + goff[j]);
                zq[d][j] = *reinterpret_cast<const unsigned short*>(zbase + lr * (size_t)(2 * gs) + goff[j]);
            }
        }
        if (!PAIR) {
#pragma unroll
            for (int t = 0; t < NKW; ++t) wk[d][t] = *reinterpret_cast<const uint32_t*>(kbase_p + lr * (size_t)(2 * k) + koff[t]);
        }
    };
    auto issue_pair = [&](int row_in) {   // ... or of the pair that starts at row_in
        if (PAIRP) {
            const size_t lr = (size_t)min(row_in + p_row, n_rows - 1);
            sq[0][0] = *reinterpret_cast<const unsigned short*>(sbase + lr * (size_t)(2 * gs) + goff[0]);
            zq[0][0] = *reinterpret_cast<const unsigned short*>(zbase + lr * (size_t)(2 * gs) + goff[0]);
        }
        if (PAIR) {
            const unsigned char* kp = kbase_p + (size_t)min(row_in + (lane >> 5), n_rows - 1) * (size_t)(2 * k) + koff[0];
            if (NKW == 1) {
                const uint2 v = *reinterpret_cast<const uint2*>(kp);
                wk[0][0] = v.x;
                wk[0][1] = v.y;
            } else {
                const u4 v = *reinterpret_cast<const u4*>(kp);
                wk[0][0] = v.x;
                wk[0][1] = v.y;
                wk[0][WKN > 2 ? 2 : 0] = v.z;
                wk[0][WKN > 2 ? 3 : 1] = v.w;
            }
        }
    };

    // ---- requests: the activations this thread stages, then the first DEPTH rows ----------------------------
    // unit u = 8 columns of the padded quantized range [0, 2048 nl_all); XU units per thread and pass
    constexpr int XU = 4;
    const int n_units = 256 * nl_all;
    u4 xv[XU];
    auto gather8 = [&](int c0) {   // 8 activations at stored columns c0 .. c0 + 7 through the table
        const u4 lo = *reinterpret_cast<const u4*>(perm + c0), hi = *reinterpret_cast<const u4*>(perm + c0 + 4);
        const unsigned short* xs = reinterpret_cast<const unsigned short*>(X);
        uint32_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = xs[min(max((int)(e < 4 ? lo[e] : hi[e - 4]), 0), ic - 1)];
        return u4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
    };
    auto load_units = [&](int base) {
#pragma unroll
        for (int t = 0; t < XU; ++t) {
            const int c0 = min(8 * (base + t * DOT_THREADS + tid), kq - 8);
            xv[t] = PERM ? gather8(c0) : *reinterpret_cast<const u4*>(X + c0);
        }
    };
    // pair order of a word's conversion: (x0, x4) (x1, x5) (x2, x6) (x3, x7); with it the unit's sums
    // sum base x (base 1024 for the pairs at bits 0..3, 64 for those at bits 4..7) and sum x, added over the four
    // units of a lane's 32 columns (threads 4 j .. 4 j + 3 of the staging pass hold them)
    float2* ksum = reinterpret_cast<float2*>(lds + 4096 * nl_all);
    unsigned char* xweak = lds + 4096 * nl_all + 512 * nl_all;
    auto quad_sum = [](float f) {
        f += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, f), 0xB1, 0xf, 0xf, false));
        f += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, f), 0x4E, 0xf, 0xf, false));
        return f;
    };
    auto store_units = [&](int base) {
#pragma unroll
        for (int t = 0; t < XU; ++t) {
            const int u = base + t * DOT_THREADS + tid;
            u4 v = xv[t];
            if (8 * u >= kq) v = u4{0u, 0u, 0u, 0u};
            u4 p;
            if (W3D) {
                p = v;   // column order; every code gets the base 1024, so "se" below is the whole sum
            } else {
                p.x = __builtin_amdgcn_perm(v.z, v.x, 0x05040100u);   // (x0, x4)   base 1024
                p.y = __builtin_amdgcn_perm(v.z, v.x, 0x07060302u);   // (x1, x5)   base 64
                p.z = __builtin_amdgcn_perm(v.w, v.y, 0x05040100u);   // (x2, x6)   base 1024
                p.w = __builtin_amdgcn_perm(v.w, v.y, 0x07060302u);   // (x3, x7)   base 64
            }
            // (copies first: a bit cast applied directly to a vector component read the first component every time)
            const uint32_t px = p.x, py = p.y, pz = p.z, pw = p.w;
            const h2 a = __builtin_bit_cast(h2, px), b = __builtin_bit_cast(h2, py), c = __builtin_bit_cast(h2, pz),
                     d = __builtin_bit_cast(h2, pw);
            const float se = quad_sum(((float)a.x + (float)a.y) + ((float)c.x + (float)c.y));
            const float so = quad_sum(((float)b.x + (float)b.y) + ((float)d.x + (float)d.y));
            if (u < n_units) {
                // range i = u / 256, lane l = (u % 256) / 4, piece q = u % 4  ->  [i][q][l]
                const int i = u >> 8, l = (u & 255) >> 2, q = u & 3;
                *reinterpret_cast<u4*>(lds + 4096 * i + 1024 * q + 16 * l) = p;
                if (q == 0) ksum[64 * i + l] = float2{1024.f * se + (W3D ? 1024.f : 64.f) * so, se + so};
            }
        }
    };
    load_units(0);
    // the weak activations: one 16-byte unit per thread (k <= 8 * DOT_THREADS)
    const u4 xwv = PERM ? gather8(kq + min(8 * tid, k - 8)) : *reinterpret_cast<const u4*>(X + kq + min(8 * tid, k - 8));
    issue_pair(row_first);   // the small requests first: they return first and nothing waits behind a kilobyte for them
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) issue_small(d, row_first + d);
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) issue_w(d, row_first + d);
    __builtin_amdgcn_sched_barrier(0);   // nothing below may move above the requests

    // ---- stage the activations --------------------------------------------------------------------------------
    store_units(0);
    if (8 * tid < k) *reinterpret_cast<u4*>(xweak + 16 * tid) = xwv;
    for (int base = XU * DOT_THREADS; base < n_units; base += XU * DOT_THREADS) {   // rows longer than 16384 columns
        load_units(base);
        store_units(base);
    }
    __syncthreads();

    // ---- this lane's activations, for the rest of the launch ----------------------------------------------------
    uint32_t xr[NL][16];
    float kbase[NL], ssum[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const u4 v = *reinterpret_cast<const u4*>(lds + 4096 * (li0 + i) + 1024 * q + 16 * lane);
            xr[i][4 * q + 0] = v.x;
            xr[i][4 * q + 1] = v.y;
            xr[i][4 * q + 2] = v.z;
            xr[i][4 * q + 3] = v.w;
        }
        const float2 ks2 = ksum[64 * (li0 + i) + lane];
        kbase[i] = ks2.x;
        ssum[i] = ks2.y;
    }
    float ssel[NP];   // sum x of the group this lane applies the parameters of set j to (0: none)
#pragma unroll
    for (int j = 0; j < NP; ++j) ssel[j] = 0.f;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const float sg = quad_sum(ssum[i]);
        if (PAIRP) {
            if (p_rng == i && qm < 2 * NL) ssel[0] = sg;
        } else {
            if (qm == (i & 3)) ssel[i >> 2] = sg;
        }
    }
    uint32_t xw[WKN];
    if (PAIR) {
        const int c0 = 4 * NKW * (lane & 31);   // columns c0 .. c0 + 4 NKW - 1 (k is a multiple of 8: whole or nothing)
#pragma unroll
        for (int t = 0; t < WKN; ++t) xw[t] = (c0 + 2 * t < k) ? *reinterpret_cast<const uint32_t*>(xweak + 2 * c0 + 4 * t) : 0u;
    } else {
#pragma unroll
        for (int t = 0; t < NKW; ++t) {
            const int dw = lane + 64 * (t * KS + kpart);
            xw[t] = (2 * dw < k) ? *reinterpret_cast<const uint32_t*>(xweak + 4 * dw) : 0u;
        }
    }

    uint32_t m_lo = 0x000f000fu, m_hi = 0x00f000f0u, g_lo = 0x64006400u, g_hi = 0x54005400u, m3 = 0x00070007u;
    asm volatile("" : "+v"(m_lo), "+v"(m_hi), "+v"(g_lo), "+v"(g_hi), "+v"(m3));   // in registers: (w & m) | g is then one v_and_or_b32

    float res = 0.f;   // lane j: the wave's result for its row j
    // sum x q of every group of one row's ranges, each in the four lanes of its quad
    auto row_sums = [&](int d, float (&tg)[NL]) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            float a0 = 0.f, a1 = 0.f;
            if (W3D) {
                const uint32_t w0 = wq[d][i].x, w1 = wq[d][i].y, w2 = wq[d][i].z;
#pragma unroll
                for (int P = 0; P < 16; ++P) {
                    constexpr uint32_t spread = 0x2001u;
                    uint32_t f;   // the pair's six bits
                    if (P < 5) f = __builtin_amdgcn_ubfe(w0, 6 * P, 6);
                    else if (P == 5) f = __builtin_amdgcn_alignbit(w1, w0, 30) & 63u;
                    else if (P < 10) f = __builtin_amdgcn_ubfe(w1, 6 * P - 32, 6);
                    else if (P == 10) f = __builtin_amdgcn_alignbit(w2, w1, 28) & 63u;
                    else f = __builtin_amdgcn_ubfe(w2, 6 * P - 64, 6);
                    const uint32_t pr = ((f * spread) & m3) | g_lo;
                    if (P & 1) a1 = dot2(pr, xr[i][P], a1);
                    else a0 = dot2(pr, xr[i][P], a0);
                }
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t w = wq[d][i][q], w8 = w >> 8;
                    const uint32_t p0 = (w & m_lo) | g_lo, p1 = (w & m_hi) | g_hi, p2 = (w8 & m_lo) | g_lo, p3 = (w8 & m_hi) | g_hi;
                    a0 = dot2(p0, xr[i][4 * q + 0], a0);
                    a1 = dot2(p1, xr[i][4 * q + 1], a1);
                    a0 = dot2(p2, xr[i][4 * q + 2], a0);
                    a1 = dot2(p3, xr[i][4 * q + 3], a1);
                }
            }
            tg[i] = quad_sum((a0 + a1) - kbase[i]);
        }
    };
    // the parameters of one row applied to its group sums (the per-row sets)
    auto row_scaled = [&](int d, const float (&tg)[NL]) {
        float tsel[NP], y = 0.f;
#pragma unroll
        for (int jj = 0; jj < NP; ++jj) tsel[jj] = 0.f;
#pragma unroll
        for (int i = 0; i < NL; ++i)
            if (qm == (i & 3)) tsel[i >> 2] = tg[i];
#pragma unroll
        for (int jj = 0; jj < NP; ++jj) {
            const float sc = (float)__builtin_bit_cast(_Float16, (unsigned short)sq[d][jj]);
            const float z = (float)__builtin_bit_cast(_Float16, (unsigned short)zq[d][jj]);
            y = fmaf(sc, fmaf(-z, ssel[jj], tsel[jj]), y);
        }
        return y;
    };
    auto finish = [&](float y, int j) {
        const float tot = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wave_sum_to_lane63(y)), 63));
        res = (lane == j) ? tot : res;
    };

    // One pair / one row; REFILL: request the next one behind it.  The last one is peeled off so that no request
    // stands under a condition (the compiler would wait for every outstanding load at the join).
    auto pair_step = [&](int b, auto refill) {
        constexpr bool REFILL = decltype(refill)::value;
        const int next = row_first + (b + 1) * 2;
        float t0[NL], t1[NL];
        row_sums(0, t0);
        if (REFILL) issue_w(0, next);
        __builtin_amdgcn_sched_barrier(0);   // keep the refill right behind its row
        row_sums(1, t1);
        if (REFILL) issue_w(1, next + 1);
        __builtin_amdgcn_sched_barrier(0);
        float y0, y1;
        if (PAIRP) {
            float tsel = 0.f;
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                if (qm == i) tsel = t0[i];
                if (qm == NL + i) tsel = t1[i];
            }
            const float sc = (float)__builtin_bit_cast(_Float16, (unsigned short)sq[0][0]);
            const float z = (float)__builtin_bit_cast(_Float16, (unsigned short)zq[0][0]);
            const float c = sc * fmaf(-z, ssel[0], tsel);
            y0 = p_row == 0 ? c : 0.f;
            y1 = p_row == 1 ? c : 0.f;
        } else {
            y0 = row_scaled(0, t0);
            y1 = row_scaled(1, t1);
        }
        float yw = 0.f;
#pragma unroll
        for (int t = 0; t < WKN; ++t) yw = dot2(wk[0][t], xw[t], yw);
        y0 += lane < 32 ? yw : 0.f;
        y1 += lane < 32 ? 0.f : yw;
        if (REFILL) {
            issue_small(0, next);
            issue_small(1, next + 1);
            issue_pair(next);
        }
        __builtin_amdgcn_sched_barrier(0);
        finish(y0, 2 * b);
        finish(y1, 2 * b + 1);
    };
    auto row_step = [&](int b, auto refill) {
        constexpr bool REFILL = decltype(refill)::value;
        float t0[NL];
        row_sums(0, t0);
        float y = row_scaled(0, t0);
#pragma unroll
        for (int t = 0; t < NKW; ++t) y = dot2(wk[0][t], xw[t], y);
        if (REFILL) {
            issue_small(0, row_first + b + 1);
            issue_w(0, row_first + b + 1);
        }
        __builtin_amdgcn_sched_barrier(0);   // keep the refill right behind its row
        finish(y, b);
    };
    if constexpr (PAIR) {
        for (int b = 0; b + 1 < B; ++b) pair_step(b, std::true_type{});
        pair_step(B - 1, std::false_type{});
    } else {
        for (int b = 0; b + 1 < B; ++b) row_step(b, std::true_type{});
        row_step(B - 1, std::false_type{});
    }

    // ---- K split: partial results meet in LDS; then one store per row ----------------------------------------------
    if (KS > 1) {
        float* xch = reinterpret_cast<float*>(xweak + 256 * KS * NKW);
        if (kpart > 0) xch[64 * wave + lane] = res;
        __syncthreads();
        if (kpart == 0)
            for (int p = 1; p < KS; ++p) res += xch[64 * (wave + p) + lane];
    }
    if (live && kpart == 0 && lane < rpw && row_first + lane < n_rows) yout[row_first + lane] = __float2half_rn(res);
}

// =============================================================================================
// Three-bit codes, ten to a 32-bit word (the canonical layout), one activation row.  Same shape as the 4-bit kernel
// above - whole rows per wave in contiguous 1 KB requests, activations in registers - with the group structure
// read off the layout: 1 KB = 256 words = 2560 codes = exactly 20 groups of 128, and a lane's 16 bytes = 40 codes
// = five chunks of 8.  Inside each run of 16 lanes (640 codes = 5 groups) the boundaries 128, 256, 384, 512 fall on
// chunk boundaries of lanes 3, 6, 9 and 12; every other lane lies in one group.  So a lane keeps five chunk sums
// (four two-element dot products each, codes as the exact fp16 numbers 1024 + q), splits them into "its first
// group" and "its second group" by a per-lane prefix select, and applies the two groups' scales and zero-points
// to those two sums: s (sum x (1024 + q) - (1024 + z) sum x).  A pair of codes never straddles words (ten per
// word): one 6-bit field extract and one multiplication by 2^13 + 1 put its codes at bits 0..2 and 16..18.
// The four parameters of a lane's two groups come with one 8-byte load per array (four consecutive groups
// starting at an even one) and one byte permute.
// LDS: activation chunks [NL][5][64 lanes] 16 B | chunk sums float [NL][5][64] | weak activations fp16 [128 NKW]
// =============================================================================================
template <int NL, int DEPTH, int NKW>
__global__ __launch_bounds__(DOT_THREADS) void gemv_w3_dot_kernel(DotLayers R, int kq, int k, int row_bytes, int gs,
                                                                   const __half* __restrict__ X, int B) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    typedef uint32_t u2 __attribute__((ext_vector_type(2)));
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rpw = DEPTH * B;
    const int sidx_raw = blockIdx.x * DOT_WAVES + wave;
    const bool live = sidx_raw < R.n_sets;
    const int sidx = min(sidx_raw, R.n_sets - 1);
    const int li = (sidx >= R.set_begin[1]) + (sidx >= R.set_begin[2]) + (sidx >= R.set_begin[3]);
    const int row_first = (sidx - R.set_begin[li]) * rpw, n_rows = R.oc[li];
    const unsigned char* const wbase = reinterpret_cast<const unsigned char*>(R.qweight[li]);
    const unsigned char* const sbase = reinterpret_cast<const unsigned char*>(R.scales[li]);
    const unsigned char* const zbase = reinterpret_cast<const unsigned char*>(R.zeros[li]);
    const unsigned char* const kbase_p = reinterpret_cast<const unsigned char*>(R.weak[li]);
    __half* const yout = R.Y[li];

    // ---- per-lane offsets; the lane's first group of range i is 20 i + 5 lane / 16, its parameters are halfs sel, sel + 1
    // of the four fetched from the even group g' <= gs - 4
    int woff[NL], goff[NL], koff[NKW];
    uint32_t selb[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        woff[i] = min(1024 * i + 16 * lane, row_bytes - 16);
        const int g_lo = 20 * i + ((5 * lane) >> 4);
        const int gp = max(min(g_lo & ~1, gs - 4), 0);
        const int sl = min(max(g_lo - gp, 0), 3), sh = min(sl + 1, 3);
        goff[i] = 2 * gp;
        selb[i] = (uint32_t)(2 * sl) | ((uint32_t)(2 * sl + 1) << 8) | ((uint32_t)(2 * sh) << 16) | ((uint32_t)(2 * sh + 1) << 24);
    }
#pragma unroll
    for (int t = 0; t < NKW; ++t) koff[t] = 4 * min(lane + 64 * t, (k >> 1) - 1);

    u4 wq[DEPTH][NL];
    u2 sq[DEPTH][NL], zq[DEPTH][NL];
    uint32_t wk[DEPTH][NKW];
    auto issue = [&](int d, int row_in) {
        const size_t lr = (size_t)min(row_in, n_rows - 1);
        const unsigned char* wrow = wbase + lr * (size_t)row_bytes;
        const unsigned char* srow = sbase + lr * (size_t)(2 * gs);
        const unsigned char* zrow = zbase + lr * (size_t)(2 * gs);
        const unsigned char* krow = kbase_p + lr * (size_t)(2 * k);
        // the small requests first: they return first and nothing waits behind a kilobyte for them
#pragma unroll
        for (int t = 0; t < NKW; ++t) wk[d][t] = *reinterpret_cast<const uint32_t*>(krow + koff[t]);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            sq[d][i] = *reinterpret_cast<const u2*>(srow + goff[i]);
            zq[d][i] = *reinterpret_cast<const u2*>(zrow + goff[i]);
        }
#pragma unroll
        for (int i = 0; i < NL; ++i) wq[d][i] = *reinterpret_cast<const u4*>(wrow + woff[i]);
    };

    // ---- requests: the activations this thread stages, then the first DEPTH rows ----------------------------
    // unit u = 8 columns: chunk u % 5 of lane position u / 5 (range (u / 5) / 64, lane (u / 5) % 64)
    constexpr int XU = 4;
    constexpr int n_units = 320 * NL;
    static_assert(n_units <= XU * DOT_THREADS, "one staging pass");
    u4 xv[XU];
#pragma unroll
    for (int t = 0; t < XU; ++t) xv[t] = *reinterpret_cast<const u4*>(X + min(8 * (t * DOT_THREADS + tid), kq - 8));
    u4 xwv = *reinterpret_cast<const u4*>(X + kq + min(8 * tid, k - 8));
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) issue(d, row_first + d);
    __builtin_amdgcn_sched_barrier(0);   // nothing below may move above the requests

    float* csum = reinterpret_cast<float*>(lds + 5120 * NL);
    unsigned char* xweak = lds + 5120 * NL + 1280 * NL;
#pragma unroll
    for (int t = 0; t < XU; ++t) {
        const int u = t * DOT_THREADS + tid;
        u4 v = xv[t];
        if (8 * u >= kq) v = u4{0u, 0u, 0u, 0u};
        const uint32_t vx = v.x, vy = v.y, vz = v.z, vw = v.w;
        const h2 a = __builtin_bit_cast(h2, vx), b = __builtin_bit_cast(h2, vy), c = __builtin_bit_cast(h2, vz), d = __builtin_bit_cast(h2, vw);
        const float su = (((float)a.x + (float)a.y) + ((float)b.x + (float)b.y)) + (((float)c.x + (float)c.y) + ((float)d.x + (float)d.y));
        if (u < n_units) {
            const int pos = u / 5, ch = u - 5 * pos, i = pos >> 6, l = pos & 63;
            *reinterpret_cast<u4*>(lds + 5120 * i + 1024 * ch + 16 * l) = v;
            csum[(5 * i + ch) * 64 + l] = su;
        }
    }
    if (8 * tid < k) *reinterpret_cast<u4*>(xweak + 16 * tid) = xwv;
    __syncthreads();

    // ---- this lane's activations and group sums, for the rest of the launch ---------------------------------------
    const int j16 = lane & 15;
    const int bc = j16 == 3 ? 1 : (j16 == 6 ? 2 : (j16 == 9 ? 3 : (j16 == 12 ? 4 : 5)));   // chunks of the lane's first group
    uint32_t xr[NL][20];
    float s_lo[NL], s_hi[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        float lo = 0.f, all = 0.f;
#pragma unroll
        for (int ch = 0; ch < 5; ++ch) {
            const u4 v = *reinterpret_cast<const u4*>(lds + 5120 * i + 1024 * ch + 16 * lane);
            xr[i][4 * ch + 0] = v.x;
            xr[i][4 * ch + 1] = v.y;
            xr[i][4 * ch + 2] = v.z;
            xr[i][4 * ch + 3] = v.w;
            const float sc = csum[(5 * i + ch) * 64 + lane];
            all += sc;
            if (ch < bc) lo += sc;
        }
        s_lo[i] = lo;
        s_hi[i] = all - lo;
    }
    uint32_t xw[NKW];
#pragma unroll
    for (int t = 0; t < NKW; ++t) {
        const int dw = lane + 64 * t;
        xw[t] = (2 * dw < k) ? *reinterpret_cast<const uint32_t*>(xweak + 4 * dw) : 0u;
    }
    uint32_t cmask = 0x00070007u, cmagic = 0x64006400u;
    asm volatile("" : "+v"(cmask), "+v"(cmagic));   // in registers: (v & m) | g is then one v_and_or_b32

    float res = 0.f;   // lane j: the wave's result for its row j
    auto compute = [&](int d, int j) {
        float y = 0.f;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            float c[5] = {0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int P = 0; P < 20; ++P) {   // pair P: codes 2 P, 2 P + 1 of the lane's 40 = pair P % 5 of word P / 5
                const uint32_t six = __builtin_amdgcn_ubfe(wq[d][i][P / 5], 6 * (P % 5), 6);
                const uint32_t cp = ((six * 0x2001u) & cmask) | cmagic;
                c[P / 4] = dot2(cp, xr[i][P], c[P / 4]);
            }
            const float p1 = c[0], p2 = p1 + c[1], p3 = p2 + c[2], p4 = p3 + c[3], all = p4 + c[4];
            const float a_lo = bc == 1 ? p1 : (bc == 2 ? p2 : (bc == 3 ? p3 : (bc == 4 ? p4 : all)));
            const float a_hi = all - a_lo;
            const h2 sp = __builtin_bit_cast(h2, __builtin_amdgcn_perm(sq[d][i].y, sq[d][i].x, selb[i]));
            const h2 zp = __builtin_bit_cast(h2, __builtin_amdgcn_perm(zq[d][i].y, zq[d][i].x, selb[i]));
            y = fmaf((float)sp.x, fmaf(-(1024.f + (float)zp.x), s_lo[i], a_lo), y);
            y = fmaf((float)sp.y, fmaf(-(1024.f + (float)zp.y), s_hi[i], a_hi), y);
        }
#pragma unroll
        for (int t = 0; t < NKW; ++t) y = dot2(wk[d][t], xw[t], y);
        const float tot = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wave_sum_to_lane63(y)), 63));
        res = (lane == j) ? tot : res;
    };

    for (int b = 0; b + 1 < B; ++b) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            compute(d, b * DEPTH + d);
            issue(d, row_first + (b + 1) * DEPTH + d);
            __builtin_amdgcn_sched_barrier(0);   // keep the refill right behind its row
        }
    }
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) compute(d, (B - 1) * DEPTH + d);

    if (live && lane < rpw && row_first + lane < n_rows) yout[row_first + lane] = __float2half_rn(res);
}

struct DotPlan {
    int nscw, depth, nkw, ks_log2, B;   // nscw: 1 KB ranges of a row per wave
    size_t lds;
    bool ok;
};

// Shapes the kernel takes, and how a launch is cut: ranges per wave from the row length (a wave keeps at most 8 x 2048
// columns of activations in registers, longer rows are split over 2 or 4 waves), two rows in flight for rows of up
// to three ranges, batches so that the row sets fill the resident waves once.
DotPlan dot_plan(const Layer& L, int n_rows) {
    DotPlan p = {};
    p.ok = false;
    const bool w3d = L.bits == 3 && L.dense;   // (the dense layout's rows hold whole 12-byte lane pieces when Kq is a multiple of 32)
    if (!(L.bits == 4 || w3d) || L.g != 128 || L.kq < 8 || (L.kq % 8) != 0 || L.k < 8 || (L.k % 8) != 0) return p;
    if (w3d && ((L.kq % 32) != 0 || L.stride < 3)) return p;
    const int nl_all = ceil_div(L.kq, 2048);
    int ks_log2 = 0;
    // one wave for rows of up to 8 ranges; longer rows over 2 waves, or over 4 when that leaves a wave at least 4 ranges
    // (28416 columns: 27.2 us with 4 x 4 ranges, two workgroups per CU, against 28.5 us with 2 x 8)
    if (nl_all > 8) ks_log2 = nl_all > 12 ? 2 : 1;
    const int KS = 1 << ks_log2;
    int nl = ceil_div(nl_all, KS);
    if (nl > 8) return p;
    nl = nl < 2 ? 2 : (nl == 7 ? 8 : nl);   // (seven ranges spill registers; the eighth is clamped and multiplies zeros)
    if (KS > 1 && nl < 4) nl = 4;           // (the variants of 2 and 3 ranges run pairs of rows and take no K split)
    const int nkw = ceil_div(L.k, 128 * KS);
    if (nkw > 2 || L.k > 8 * DOT_THREADS) return p;
    p.nscw = nl;
    p.nkw = nkw;
    p.ks_log2 = ks_log2;
    p.depth = (nl <= 3 && KS == 1) ? 2 : 1;
    const int occ_wg = nl <= 4 ? 2 : 1;                         // resident workgroups per CU the register budget allows (87 / 119 / 116 registers at 2 / 3 / 4 ranges)
    const int slots = 256 * occ_wg * (DOT_WAVES / KS);          // row sets resident at once
    p.B = ceil_div(n_rows, p.depth * slots);
    if (p.depth * p.B > 64) return p;                           // a wave keeps its rows' results one per lane
    const int nl_pad = nl * KS;
    p.lds = (size_t)4096 * nl_pad + 512 * nl_pad + 256 * KS * nkw + (KS > 1 ? DOT_WAVES * 64 * sizeof(float) : 0);
    p.ok = p.lds <= 80 * 1024;
    return p;
}

// The 3-bit kernel: nscw holds NL, the 1 KB ranges of a row (at most 6: 15360 columns); no K split, no gather.
DotPlan dot_plan_w3(const Layer& L, int n_rows, bool perm) {
    DotPlan p = {};
    p.ok = false;
    if (perm || L.bits != 3 || L.dense || L.g != 128 || L.kq < 8 || (L.kq % 8) != 0 || L.k < 8 || (L.k % 8) != 0 || L.gs < 8) return p;
    const int nl = ceil_div(L.stride, 256);
    if (nl > 6) return p;
    const int nkw = ceil_div(L.k, 128);
    if (nkw > 2) return p;
    p.nscw = nl;
    p.nkw = nkw;
    p.ks_log2 = 0;
    p.depth = nl <= 2 ? 2 : 1;
    const int occ_wg = nl <= 2 ? 2 : 1;
    const int slots = 256 * occ_wg * DOT_WAVES;
    p.B = ceil_div(n_rows, p.depth * slots);
    if (p.depth * p.B > 64) return p;
    p.lds = (size_t)5120 * nl + 1280 * nl + 256 * nkw;
    p.ok = p.lds <= 64 * 1024;
    return p;
}

using DotKern = void (*)(DotLayers, int, int, int, int, const __half*, const int*, int, int, int);

template <bool PERM, bool W3D>
DotKern dot_kernel(int nl, int nkw) {
#define QEFT_DOT(N, D) (nkw == 1 ? (DotKern)gemv_w4_dot_kernel<N, D, 1, PERM, W3D> : (DotKern)gemv_w4_dot_kernel<N, D, 2, PERM, W3D>)
    switch (nl) {
        case 2: return QEFT_DOT(2, 2);
        case 3: return QEFT_DOT(3, 2);
        case 4: return QEFT_DOT(4, 1);
        case 5: return QEFT_DOT(5, 1);
        case 6: return QEFT_DOT(6, 1);
        default: return QEFT_DOT(8, 1);
    }
#undef QEFT_DOT
}

}  // namespace

// Layers Ls[0 .. n) share the input (same IC, k, bits, group size).  *handled = false, nothing launched, when
// the shapes do not fit this kernel.
hipError_t gemv_dot_fwd(const Layer* Ls, int n, const int* perm, const __half* X, __half* const* Y, hipStream_t s, bool* handled) {
    *handled = false;
    if (n < 1 || n > MAX_GROUP) return hipSuccess;
    DotLayers R = {};
    int rows = 0;
    for (int i = 0; i < n; ++i) rows += Ls[i].oc;
    const Layer& L = Ls[0];
    const bool w3 = L.bits == 3 && !L.dense;
    DotPlan p = w3 ? dot_plan_w3(L, rows, perm != nullptr) : dot_plan(L, rows);
    if (!p.ok) return hipSuccess;
    const int rpw = p.depth * p.B;
    int sets = 0;
    for (int i = 0; i < MAX_GROUP; ++i) {
        const Layer& Li = Ls[i < n ? i : 0];
        R.qweight[i] = Li.qweight;
        R.scales[i] = Li.scales;
        R.zeros[i] = Li.zeros;
        R.weak[i] = Li.weak;
        R.Y[i] = Y[i < n ? i : 0];
        R.oc[i] = Li.oc;
        R.set_begin[i] = i < n ? sets : INT_MAX;
        if (i < n) sets += ceil_div(Li.oc, rpw);
    }
    R.n_sets = sets;
    if (w3) {
        using W3Kern = void (*)(DotLayers, int, int, int, int, const __half*, int);
#define QEFT_W3(N, D) (p.nkw == 1 ? (W3Kern)gemv_w3_dot_kernel<N, D, 1> : (W3Kern)gemv_w3_dot_kernel<N, D, 2>)
        const W3Kern k3 = p.nscw == 1 ? QEFT_W3(1, 2) : (p.nscw == 2 ? QEFT_W3(2, 2) : (p.nscw == 3 ? QEFT_W3(3, 1) : (p.nscw == 4 ? QEFT_W3(4, 1) : (p.nscw == 5 ? QEFT_W3(5, 1) : QEFT_W3(6, 1)))));
#undef QEFT_W3
        k3<<<ceil_div(sets, DOT_WAVES), DOT_THREADS, p.lds, s>>>(R, L.kq, L.k, 4 * L.stride, L.gs, X, p.B);
        *handled = true;
        return hipGetLastError();
    }
    const int blocks = ceil_div(sets, DOT_WAVES >> p.ks_log2);
    if (L.dense && perm) return hipSuccess;   // no gathering variant for 3-bit codes
    const DotKern kern = L.dense ? dot_kernel<false, true>(p.nscw, p.nkw) : (perm ? dot_kernel<true, false>(p.nscw, p.nkw) : dot_kernel<false, false>(p.nscw, p.nkw));
    if (p.lds > 64 * 1024) {   // (rows of more than 24 K columns; idempotent, so set on every such launch)
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
        if (e != hipSuccess) return e;
    }
    kern<<<blocks, DOT_THREADS, p.lds, s>>>(R, L.kq, L.k, 4 * L.stride, L.gs, X, perm, L.ic, p.B, p.ks_log2);
    *handled = true;
    return hipGetLastError();
}

}  // namespace qeft
