// Shared pieces of the tiled MFMA GEMM kernels (forward, input gradient, weak-column gradient).
//
// A workgroup of 4 waves owns a 256 x 256 output tile C[i][j] = sum_k A[i][k] * B[j][k]; each
// wave 128 x 128 (4 x 4 MFMA 32x32x16 tiles) in the LDS-staged kernels, 64 x 256 (2 x 8) in the
// register-operand kernels - 256 fp32 accumulators per lane either way.  K advances
// in stages of 64: both operand tiles are 256 rows x 64 halfs in LDS, rows of 128 bytes whose
// 16-byte chunks are XOR-swizzled with the row number so that fragment reads and the producers'
// writes are free of bank conflicts; two buffers per operand (128 KB of the CU's 160 KB).
// The operand roles are chosen per kernel so that "i" runs along the contiguous dimension of
// the result: a lane owns 4 consecutive i for one j, i.e. 8 (fp16) or 16 (fp32) contiguous bytes.
#pragma once

#include "qeft_internal.h"

namespace qeft {
namespace gemm {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));

constexpr int BT = 256;                  // tile rows of either operand
constexpr int BK = 64;                   // K per stage
constexpr int TILE_BYTES = BT * BK * 2;  // 32 KB
constexpr int GEMM_LDS = 4 * TILE_BYTES; // A0 A1 B0 B1

__device__ __forceinline__ u4 ld16(const void* p) { return *reinterpret_cast<const u4*>(p); }
__device__ __forceinline__ uint32_t h2_bits(h2 v) { return __builtin_bit_cast(uint32_t, v); }
__device__ __forceinline__ h2 bits_h2(uint32_t v) { return __builtin_bit_cast(h2, v); }

// Byte offset of 16-byte chunk `c` (0..7) of row `r` inside a 256 x 64 half tile.  A row is one
// 128-byte line = one pass over the LDS banks, which a 128-bit access makes with 8 lanes at a
// time.  The chunk slot is XOR-ed with row bits 0..2 and 3..5 so that 8 neighbouring lanes hit 8
// different slots in every access pattern the kernels use: fragment reads (8 consecutive rows, one
// chunk), row-wise producer stores (one row x 8 chunks, or 4 rows x 2 half-rows) and transposing
// producer stores (rows 8 apart, one chunk).  (Measured: SQ_LDS_BANK_CONFLICT.)
__device__ __forceinline__ int tile_off(int r, int c) { return r * 128 + ((c ^ (r & 7) ^ ((r >> 3) & 7)) << 4); }

// The two constants of the code -> fp16 conversion in vector registers the compiler cannot
// see through, so that (w & mask) | magic selects the single v_and_or_b32.
struct Consts {
    uint32_t mask, magic;
};
__device__ __forceinline__ Consts make_consts() {
    Consts c{0x000f000fu, 0x64006400u};
    asm volatile("" : "+v"(c.mask), "+v"(c.magic));
    return c;
}

// two codes (as 1024 + q in packed fp16) -> two weights: ((h - 1024) - z) * s.  The first
// subtraction is exact, the second rounds once (exact for integer zero-points), the product once.
__device__ __forceinline__ uint32_t dequant_pair(uint32_t hbits, h2 z2, h2 s2) {
    const h2 k1024 = h2{(_Float16)1024.f, (_Float16)1024.f};
    return h2_bits(((bits_h2(hbits) - k1024) - z2) * s2);
}

// 8 halfs x0..x7 -> (x0,x4)(x1,x5)(x2,x6)(x3,x7): the order nibbles leave the mask-and-or conversion
__device__ __forceinline__ u4 permute_x(u4 v) {
    u4 r;
    r.x = __builtin_amdgcn_perm(v.z, v.x, 0x05040100u);
    r.y = __builtin_amdgcn_perm(v.z, v.x, 0x07060302u);
    r.z = __builtin_amdgcn_perm(v.w, v.y, 0x05040100u);
    r.w = __builtin_amdgcn_perm(v.w, v.y, 0x07060302u);
    return r;
}

// 8 x 8 half transpose in registers: in[e] holds 8 consecutive columns of row e; out[j] holds
// column j of the 8 rows (rows ascending).
__device__ __forceinline__ void transpose8x8(const u4 (&in)[8], u4 (&out)[8]) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
#pragma unroll
        for (int p = 0; p < 4; ++p) out[j][p] = __builtin_amdgcn_perm(in[2 * p + 1][j >> 1], in[2 * p][j >> 1], sel);
    }
}

// XCD-aware tile order.  Workgroup b runs on XCD b % 8, and each XCD has its own L2.  Tile v of
// a row-major (slow index = activation panel) enumeration goes to the workgroup (v % per_xcd) * 8
// + v / per_xcd, so that every XCD walks a contiguous range of tiles: the 32 workgroups resident
// on an XCD then share one or two activation panels in that XCD's L2 instead of sixteen.
// The grid is 8 * per_xcd workgroups; returns -1 for the few that have no tile.
constexpr int N_XCD = 8;
__device__ __forceinline__ int xcd_tile(int n_tiles) {
    const int per_xcd = (n_tiles + N_XCD - 1) / N_XCD;
    const int v = (int)(blockIdx.x % N_XCD) * per_xcd + (int)(blockIdx.x / N_XCD);
    return v < n_tiles ? v : -1;
}
inline int xcd_grid(int n_tiles) { return N_XCD * ((n_tiles + N_XCD - 1) / N_XCD); }

// Tile index -> (weight tile t_n, activation panel t_m).  Panels are taken in bands of TILE_BAND: inside a band the
// panel index runs fastest, so the 32 consecutive tiles that are resident on an XCD at a time cover TILE_BAND panels x
// 32 / TILE_BAND weight tiles instead of one panel x 32 weight tiles.  With 4-bit weights a weight tile holds a quarter
// of a panel's bytes, and two panels x 16 weight tiles is what an XCD's L2 has to fetch least for per round of tiles.
#ifndef QEFT_TILE_BAND
#define QEFT_TILE_BAND 4
#endif
__device__ __forceinline__ void tile_coords(int tile, int tiles_n, int tiles_m, int& t_n, int& t_m) {
    constexpr int P = QEFT_TILE_BAND;
    const int band = tile / (P * tiles_n), r = tile - band * (P * tiles_n);
    const int pb = min(P, tiles_m - band * P);
    t_n = r / pb;
    t_m = band * P + (r - t_n * pb);
}

// Tile order of a launch in which some tiles are split `splits` ways along the contraction (a workgroup per split, each
// storing a partial tile of BT x BT halves into slot `slot` of a workspace; a second kernel adds them).
//   tail_first <= 0: every tile is split (launches of few tiles); order as xcd_tile over tiles * splits.
//   tail_first  > 0: each XCD walks its contiguous range of ceil(tiles / 8) tiles as in xcd_tile; the first tail_first of
//     them (whole rounds of the XCD's 32 CUs) are not split, the rest - the last, partly filled round - are, all splits
//     of one index after the other.  Slots number the tail tiles XCD by XCD.
// Returns false for a workgroup without work; slot < 0 for a tile that is not split.
__device__ __forceinline__ bool split_tile(int tiles_all, int tail_first, int splits, int& tile, int& sp, int& slot) {
    if (tail_first <= 0) {
        const int v = xcd_tile(tiles_all * splits);
        if (v < 0) return false;
        sp = v / tiles_all;
        tile = v - sp * tiles_all;
        slot = splits > 1 ? tile * splits + sp : -1;
        return true;
    }
    const int per = (tiles_all + N_XCD - 1) / N_XCD;
    const int x = (int)(blockIdx.x % N_XCD), l = (int)(blockIdx.x / N_XCD);
    const int tf = min(tail_first, per), ntail = per - tf;
    if (l < tf) {
        tile = x * per + l;
        sp = 0;
        slot = -1;
    } else {
        const int j = l - tf;
        sp = j / ntail;
        const int r = j - sp * ntail;
        tile = x * per + tf + r;
        slot = (x * ntail + r) * splits + sp;
    }
    return tile < tiles_all;
}
// host side of the same order: workgroups in the grid, and partial-tile slots
inline int split_grid(int tiles_all, int tail_first, int splits) {
    if (tail_first <= 0) return xcd_grid(tiles_all * splits);
    const int per = (tiles_all + N_XCD - 1) / N_XCD, tf = tail_first < per ? tail_first : per;
    return N_XCD * (tf + (per - tf) * splits);
}
inline int split_tail_tiles(int tiles_all, int tail_first) {   // tail tiles, counting the empty ones of a ragged last XCD
    if (tail_first <= 0) return tiles_all;
    const int per = (tiles_all + N_XCD - 1) / N_XCD, tf = tail_first < per ? tail_first : per;
    return N_XCD * (per - tf);
}
// tile of tail index tt (the inverse of the slot numbering), -1 if none
__device__ __forceinline__ int split_tail_tile(int tiles_all, int tail_first, int tt) {
    if (tail_first <= 0) return tt < tiles_all ? tt : -1;
    const int per = (tiles_all + N_XCD - 1) / N_XCD;
    const int tf = min(tail_first, per), ntail = per - tf;
    const int x = tt / ntail, r = tt - x * ntail;
    const int tile = x * per + tf + r;
    return (x < N_XCD && tile < tiles_all) ? tile : -1;
}

__device__ __forceinline__ void zero_acc(f16v (&acc)[4][4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
}

// The 64 MFMAs of one stage for wave (wm, wn).
__device__ __forceinline__ void compute_stage(const unsigned char* sA, const unsigned char* sB, f16v (&acc)[4][4], int wm,
                                              int wn, int lane) {
    const int fr = lane & 31, fk = lane >> 5;  // fragment row within a 32-row MFMA tile, k half
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
            for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
}

// The same, split so that a caller can interleave other work between the four k blocks of a stage.
struct Frags {
    h8 a[4], b[4];
};
__device__ __forceinline__ void load_frags(Frags& f, const unsigned char* sA, const unsigned char* sB, int wm, int wn,
                                           int lane, int ks) {
    const int fr = lane & 31, fk = lane >> 5;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f.a[i] = *reinterpret_cast<const h8*>(sA + tile_off(wm * 128 + i * 32 + fr, 2 * ks + fk));
        f.b[i] = *reinterpret_cast<const h8*>(sB + tile_off(wn * 128 + i * 32 + fr, 2 * ks + fk));
    }
}
__device__ __forceinline__ void mfma_block(const Frags& f, f16v (&acc)[4][4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
}

// Generic wave tile of TI x TJ MFMA tiles whose first rows in the operand tiles are ra0 / rb0.
template <int TI, int TJ>
struct FragsT {
    h8 a[TI], b[TJ];
};
template <int TI, int TJ>
__device__ __forceinline__ void load_frags_t(FragsT<TI, TJ>& f, const unsigned char* sA, const unsigned char* sB, int ra0,
                                             int rb0, int lane, int ks) {
    const int fr = lane & 31, fk = lane >> 5;
#pragma unroll
    for (int i = 0; i < TI; ++i) f.a[i] = *reinterpret_cast<const h8*>(sA + tile_off(ra0 + i * 32 + fr, 2 * ks + fk));
#pragma unroll
    for (int j = 0; j < TJ; ++j) f.b[j] = *reinterpret_cast<const h8*>(sB + tile_off(rb0 + j * 32 + fr, 2 * ks + fk));
}
template <int TI, int TJ>
__device__ __forceinline__ void mfma_block_t(const FragsT<TI, TJ>& f, f16v (&acc)[TI][TJ]) {
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
}
// fp16 epilogue of such a wave tile: out[j][i], i0/j0 = global index of the wave tile's first row of A / B
template <int TI, int TJ>
__device__ __forceinline__ void store_f16_t(const f16v (&acc)[TI][TJ], __half* out, int64_t ld, int i0, int ni, int j0,
                                            int nj, int lane) {
    const int fr = lane & 31, fk = lane >> 5;
#pragma unroll
    for (int tj = 0; tj < TJ; ++tj) {
        const int j = j0 + tj * 32 + fr;
        if (j >= nj) continue;
#pragma unroll
        for (int ti = 0; ti < TI; ++ti) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int i = i0 + ti * 32 + 8 * g + 4 * fk;
                if (i < ni) {
                    const h2 lo = h2{(_Float16)acc[ti][tj][4 * g + 0], (_Float16)acc[ti][tj][4 * g + 1]};
                    const h2 hi = h2{(_Float16)acc[ti][tj][4 * g + 2], (_Float16)acc[ti][tj][4 * g + 3]};
                    *reinterpret_cast<u2*>(out + (size_t)j * ld + i) = u2{h2_bits(lo), h2_bits(hi)};
                }
            }
        }
    }
}

// Producer of an operand tile whose k dimension is contiguous in memory: row r of the tile is
// src[(row0 + r) * ld + col0 ...], 64 columns per stage.  Thread t takes chunks t + 256*u.
struct RowLoader {
    u4 v[8];
    template <class Valid>
    __device__ __forceinline__ void load(const __half* src, int64_t ld, int row0, int nrows, int col0, int ncols, int tid,
                                         Valid clamp_rows) {
        const u4 zero4 = u4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int idx = tid + 256 * u, r = idx >> 3, c = idx & 7;
            const int col = col0 + 8 * c;
            int row = row0 + r;
            bool ok = col < ncols;
            if (clamp_rows) row = min(row, nrows - 1); else ok = ok && row < nrows;
            v[u] = ok ? ld16(src + (size_t)row * ld + col) : zero4;
        }
    }
    __device__ __forceinline__ void store(unsigned char* tile, int tid, bool permute) const {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int idx = tid + 256 * u, r = idx >> 3, c = idx & 7;
            *reinterpret_cast<u4*>(tile + tile_off(r, c)) = permute ? permute_x(v[u]) : v[u];
        }
    }
};

// Producer of an operand tile whose k dimension is the ROW index of a row-major matrix:
// tile row i, stage column kk is src[(k0 + kk) * ld + i0 + i].  Thread (ko = t / 32, io = t % 32)
// loads an 8 x 8 block and transposes it in registers.
struct ColLoader {
    u4 v[8];
    __device__ __forceinline__ void load(const __half* src, int64_t ld, int k0, int k_end, int i0, int i_end, int tid) {
        const u4 zero4 = u4{0u, 0u, 0u, 0u};
        const int ko = tid >> 5, io = tid & 31;
        const int col = i0 + 8 * io;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int k = k0 + 8 * ko + e;
            v[e] = (k < k_end && col < i_end) ? ld16(src + (size_t)k * ld + col) : zero4;
        }
    }
    __device__ __forceinline__ void store(unsigned char* tile, int tid) const {
        const int ko = tid >> 5, io = tid & 31;
        u4 t[8];
        transpose8x8(v, t);
#pragma unroll
        for (int j = 0; j < 8; ++j) *reinterpret_cast<u4*>(tile + tile_off(8 * io + j, ko)) = t[j];
    }
};

// Epilogue for fp16 results out[j][i]: accumulator element 4*g + r of a lane is i = 8*g + 4*(lane/32) + r,
// j = lane % 32 of its 32 x 32 tile.  ni must be a multiple of 4.
__device__ __forceinline__ void store_f16(const f16v (&acc)[4][4], __half* out, int64_t ld, int i0, int ni, int j0, int nj,
                                          int wm, int wn, int lane) {
    const int fr = lane & 31, fk = lane >> 5;
#pragma unroll
    for (int tj = 0; tj < 4; ++tj) {
        const int j = j0 + wn * 128 + tj * 32 + fr;
        if (j >= nj) continue;
#pragma unroll
        for (int ti = 0; ti < 4; ++ti) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int i = i0 + wm * 128 + ti * 32 + 8 * g + 4 * fk;
                if (i < ni) {
                    const h2 lo = h2{(_Float16)acc[ti][tj][4 * g + 0], (_Float16)acc[ti][tj][4 * g + 1]};
                    const h2 hi = h2{(_Float16)acc[ti][tj][4 * g + 2], (_Float16)acc[ti][tj][4 * g + 3]};
                    *reinterpret_cast<u2*>(out + (size_t)j * ld + i) = u2{h2_bits(lo), h2_bits(hi)};
                }
            }
        }
    }
}

// Same for fp32 results (16-byte stores).
__device__ __forceinline__ void store_f32(const f16v (&acc)[4][4], float* out, int64_t ld, int i0, int ni, int j0, int nj,
                                          int wm, int wn, int lane) {
    const int fr = lane & 31, fk = lane >> 5;
#pragma unroll
    for (int tj = 0; tj < 4; ++tj) {
        const int j = j0 + wn * 128 + tj * 32 + fr;
        if (j >= nj) continue;
#pragma unroll
        for (int ti = 0; ti < 4; ++ti) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int i = i0 + wm * 128 + ti * 32 + 8 * g + 4 * fk;
                if (i < ni)
                    *reinterpret_cast<f4*>(out + (size_t)j * ld + i) =
                        f4{acc[ti][tj][4 * g + 0], acc[ti][tj][4 * g + 1], acc[ti][tj][4 * g + 2], acc[ti][tj][4 * g + 3]};
            }
        }
    }
}

// fp16 epilogue through LDS: the wave's 128 x 128 results are transposed through 32 KB of LDS of
// its own (rows j of 256 bytes, 16-byte chunks XOR-swizzled with j) so that the global stores are
// 16 bytes per lane and 256 contiguous bytes per row instead of 8-byte pieces of 32 different
// rows.  QUADS = false: accumulator tile t_i row 8 g + 4 fk + e is i = 32 t_i + row; QUADS =
// true: it is i = 4 row + t_i (the input-gradient kernel's quantized halves).  i0 / j0: global
// index of the wave's first i / j; i0 and ni must be multiples of 8.  The LDS region needs no
// barrier: only this wave touches it, and a wave's LDS accesses complete in order.
template <bool QUADS>
__device__ __forceinline__ void store_f16_lds(const f16v (&acc)[4][4], unsigned char* stage, __half* out, int64_t ld, int i0,
                                              int ni, int j0, int nj, int lane) {
    const int fr = lane & 31, fk = lane >> 5;
    auto pack = [](float a, float b) { return h2_bits(h2{(_Float16)a, (_Float16)b}); };
#pragma unroll
    for (int tj = 0; tj < 4; ++tj) {
        unsigned char* row = stage + (tj * 32 + fr) * 256;
        const int sw = fr & 15;
        if (!QUADS) {
#pragma unroll
            for (int ti = 0; ti < 4; ++ti)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    *reinterpret_cast<u2*>(row + (((4 * ti + g) ^ sw) << 4) + 8 * fk) =
                        u2{pack(acc[ti][tj][4 * g + 0], acc[ti][tj][4 * g + 1]), pack(acc[ti][tj][4 * g + 2], acc[ti][tj][4 * g + 3])};
        } else {
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    *reinterpret_cast<u2*>(row + (((4 * g + 2 * fk + (e >> 1)) ^ sw) << 4) + 8 * (e & 1)) =
                        u2{pack(acc[0][tj][4 * g + e], acc[1][tj][4 * g + e]), pack(acc[2][tj][4 * g + e], acc[3][tj][4 * g + e])};
        }
    }
    const int c = lane & 15, r4 = lane >> 4;
    const int i = i0 + 8 * c;
#pragma unroll 8
    for (int it = 0; it < 32; ++it) {
        const int r = 4 * it + r4;
        const u4 v = *reinterpret_cast<const u4*>(stage + r * 256 + ((c ^ (r & 15)) << 4));
        if (j0 + r < nj && i < ni) *reinterpret_cast<u4*>(out + (size_t)(j0 + r) * ld + i) = v;
    }
}

}  // namespace gemm
}  // namespace qeft
