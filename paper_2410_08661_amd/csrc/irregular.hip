// Weak columns at arbitrary input channels (paper Sec. 3.2, last paragraph; Limitations): the
// attention output projection cannot be reordered offline, so its stored form keeps the
// non-weak channels in ascending order followed by the weak block, and the activations are
// brought into that order on the fly.  Here that is a gather of X (and a scatter of dX)
// through a caller-provided workspace, around the kernels of the reordered layer:
//     Xs[m][j] = X[m][perm[j]]          dX[m][perm[j]] = dXs[m][j]
// perm (int32 [IC], device) holds the original channel of every stored column.  Entries are
// clamped to [0, IC) so that a malformed table can give wrong numbers but no access outside
// the matrices.  (The forward for M <= 4 does not come here: the matrix-vector kernel gathers
// its activations itself.)
#include "qeft_internal.h"

namespace qeft {
namespace {

typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef int i4 __attribute__((ext_vector_type(4)));

// A workgroup takes whole rows, one after the other: the row is copied into LDS with 16-byte
// loads, then every thread assembles 8 stored columns from 2-byte LDS reads through the table
// and stores them as 16 bytes (rows of up to 32 K channels fit; longer ones take the kernel
// below).  Table entries are re-read per row; they stay in L1 / L2.
constexpr int ROW_LDS_MAX = 64 * 1024;

__global__ __launch_bounds__(256) void gather_rows_kernel(const unsigned short* __restrict__ X, int M, int64_t ldx,
                                                          const int* __restrict__ perm, int ic, int chunks,
                                                          unsigned short* __restrict__ Xs, int64_t lds_, int rows_per_wg) {
    extern __shared__ __attribute__((aligned(16))) unsigned short rowbuf[];
    const int m0 = blockIdx.x * rows_per_wg;
    const int full = ic >> 3;   // whole 16-byte chunks of a source row
    for (int m = m0; m < min(m0 + rows_per_wg, M); ++m) {
        const unsigned short* row = X + (size_t)m * ldx;
        for (int c = threadIdx.x; c < full; c += 256) *reinterpret_cast<u4*>(rowbuf + 8 * c) = *reinterpret_cast<const u4*>(row + 8 * c);
        for (int j = 8 * full + threadIdx.x; j < ic; j += 256) rowbuf[j] = row[j];
        __syncthreads();
        for (int c = threadIdx.x; c < chunks; c += 256) {
            uint32_t v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int j = 8 * c + e;
                v[e] = j < ic ? rowbuf[min(max(perm[min(j, ic - 1)], 0), ic - 1)] : 0u;
            }
            *reinterpret_cast<u4*>(Xs + (size_t)m * lds_ + 8 * c) = u4{v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16)};
        }
        __syncthreads();
    }
}

// The reverse: stored columns are dropped into an LDS row at their original channels, and the
// row leaves with 16-byte stores.  Channels that no table entry names (none, for a
// permutation) receive unspecified values.
__global__ __launch_bounds__(256) void scatter_rows_kernel(const unsigned short* __restrict__ Ds, int M, int64_t ldd,
                                                           const int* __restrict__ perm, int ic, int chunks,
                                                           unsigned short* __restrict__ dX, int64_t lddx, int rows_per_wg) {
    extern __shared__ __attribute__((aligned(16))) unsigned short rowbuf[];
    const int m0 = blockIdx.x * rows_per_wg;
    const int full = ic >> 3;
    for (int m = m0; m < min(m0 + rows_per_wg, M); ++m) {
        unsigned short* row = dX + (size_t)m * lddx;
        for (int c = threadIdx.x; c < chunks; c += 256) {
            const u4 v = *reinterpret_cast<const u4*>(Ds + (size_t)m * ldd + 8 * c);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int j = 8 * c + e;
                if (j < ic) rowbuf[min(max(perm[j], 0), ic - 1)] = (unsigned short)(v[e >> 1] >> (16 * (e & 1)));
            }
        }
        __syncthreads();
        for (int c = threadIdx.x; c < full; c += 256) *reinterpret_cast<u4*>(row + 8 * c) = *reinterpret_cast<const u4*>(rowbuf + 8 * c);
        for (int j = 8 * full + threadIdx.x; j < ic; j += 256) row[j] = rowbuf[j];
        __syncthreads();
    }
}

// Rows of up to 8 K channels: the same, with this thread's table entries held in registers for all rows of
// the workgroup (NC chunks of 8 columns per thread), two row buffers so that one barrier per row suffices,
// and the next row's 16-byte loads in flight while the current one is assembled.
template <int NC>
__global__ __launch_bounds__(256) void gather_rows_reg_kernel(const unsigned short* __restrict__ X, int M, int64_t ldx,
                                                              const int* __restrict__ perm, int ic, int chunks,
                                                              unsigned short* __restrict__ Xs, int64_t lds_, int rows_per_wg) {
    extern __shared__ __attribute__((aligned(16))) unsigned short rowbuf[];   // [2][8 * chunks]
    const int pitch = 8 * chunks;
    int p[NC][8];
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        const int c = threadIdx.x + 256 * i;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int j = 8 * c + e;
            p[i][e] = j < ic ? min(max(perm[j], 0), ic - 1) : -1;
        }
    }
    const int m0 = blockIdx.x * rows_per_wg, m1 = min(m0 + rows_per_wg, M);
    u4 nxt[NC];
    auto fetch = [&](int m) {   // chunk indices are clamped, not tested: the loads stay straight-line (ldx >= 8 * chunks)
        const unsigned short* row = X + (size_t)m * ldx;
#pragma unroll
        for (int i = 0; i < NC; ++i) nxt[i] = *reinterpret_cast<const u4*>(row + 8 * min((int)threadIdx.x + 256 * i, chunks - 1));
    };
    if (m0 < m1) fetch(m0);
    for (int m = m0; m < m1; ++m) {
        unsigned short* buf = rowbuf + ((m - m0) & 1) * pitch;
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            const int c = threadIdx.x + 256 * i;
            if (c < chunks) *reinterpret_cast<u4*>(buf + 8 * c) = nxt[i];
        }
        fetch(min(m + 1, m1 - 1));
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            const int c = threadIdx.x + 256 * i;
            if (c < chunks) {
                uint32_t v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = p[i][e] >= 0 ? buf[p[i][e]] : 0u;
                *reinterpret_cast<u4*>(Xs + (size_t)m * lds_ + 8 * c) = u4{v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16)};
            }
        }
        // the buffer written two rows later is this one: every thread passes the next row's barrier first
    }
}

template <int NC>
__global__ __launch_bounds__(256) void scatter_rows_reg_kernel(const unsigned short* __restrict__ Ds, int M, int64_t ldd,
                                                               const int* __restrict__ perm, int ic, int chunks,
                                                               unsigned short* __restrict__ dX, int64_t lddx, int rows_per_wg) {
    extern __shared__ __attribute__((aligned(16))) unsigned short rowbuf[];   // [2][8 * chunks]
    const int pitch = 8 * chunks, full = ic >> 3;
    int p[NC][8];
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        const int c = threadIdx.x + 256 * i;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int j = 8 * c + e;
            p[i][e] = j < ic ? min(max(perm[j], 0), ic - 1) : -1;
        }
    }
    const int m0 = blockIdx.x * rows_per_wg, m1 = min(m0 + rows_per_wg, M);
    u4 nxt[NC];
    auto fetch = [&](int m) {
        const unsigned short* row = Ds + (size_t)m * ldd;
#pragma unroll
        for (int i = 0; i < NC; ++i) nxt[i] = *reinterpret_cast<const u4*>(row + 8 * min((int)threadIdx.x + 256 * i, chunks - 1));
    };
    if (m0 < m1) fetch(m0);
    for (int m = m0; m < m1; ++m) {
        unsigned short* buf = rowbuf + ((m - m0) & 1) * pitch;
        unsigned short* row = dX + (size_t)m * lddx;
#pragma unroll
        for (int i = 0; i < NC; ++i)
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (p[i][e] >= 0) buf[p[i][e]] = (unsigned short)(nxt[i][e >> 1] >> (16 * (e & 1)));
        fetch(min(m + 1, m1 - 1));
        __syncthreads();
        for (int c = threadIdx.x; c < full; c += 256) *reinterpret_cast<u4*>(row + 8 * c) = *reinterpret_cast<const u4*>(buf + 8 * c);
        for (int j = 8 * full + threadIdx.x; j < ic; j += 256) row[j] = buf[j];
    }
}

// Rows too long for LDS: one thread per 8 stored columns of one row, two 16-byte reads of the
// table, eight 2-byte accesses to the row.
__global__ __launch_bounds__(256) void gather_cols_kernel(const unsigned short* __restrict__ X, int M, int64_t ldx,
                                                          const int* __restrict__ perm, int ic, int chunks,
                                                          unsigned short* __restrict__ Xs, int64_t lds_) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= (int64_t)M * chunks) return;
    const int m = (int)(t / chunks), c = (int)(t % chunks);
    const unsigned short* row = X + (size_t)m * ldx;
    unsigned short v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int j = 8 * c + e;
        const int src = j < ic ? min(max(perm[j], 0), ic - 1) : 0;
        v[e] = j < ic ? row[src] : (unsigned short)0;
    }
    u4 o;
#pragma unroll
    for (int p = 0; p < 4; ++p) o[p] = (uint32_t)v[2 * p] | ((uint32_t)v[2 * p + 1] << 16);
    *reinterpret_cast<u4*>(Xs + (size_t)m * lds_ + 8 * c) = o;
}

__global__ __launch_bounds__(256) void scatter_cols_kernel(const unsigned short* __restrict__ Ds, int M, int64_t ldd,
                                                           const int* __restrict__ perm, int ic, int chunks,
                                                           unsigned short* __restrict__ dX, int64_t lddx) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= (int64_t)M * chunks) return;
    const int m = (int)(t / chunks), c = (int)(t % chunks);
    const u4 v = *reinterpret_cast<const u4*>(Ds + (size_t)m * ldd + 8 * c);
    unsigned short* row = dX + (size_t)m * lddx;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int j = 8 * c + e;
        if (j < ic) row[min(max(perm[j], 0), ic - 1)] = (unsigned short)(v[e >> 1] >> (16 * (e & 1)));
    }
}

// rows per workgroup: enough workgroups for every CU a few times over, whole rows each
inline int rows_per_wg(int64_t M) { return M >= 4096 ? 4 : (M >= 1024 ? 2 : 1); }

}  // namespace

size_t irregular_workspace(int ic, int64_t M) { return (size_t)M * (size_t)((ic + 7) / 8 * 8) * sizeof(__half); }

hipError_t gather_cols(const __half* X, int64_t M, int64_t ldx, const int* perm, int ic, __half* Xs, int64_t ldo, hipStream_t s) {
    const int chunks = (ic + 7) / 8;   // ldo >= 8 * chunks, a multiple of 8
    const int row_bytes = chunks * 16;
    if (chunks <= 1024 && (ic & 7) == 0 && (ldx & 7) == 0 && ((uintptr_t)X & 15) == 0) {   // whole 16-byte chunks only: no read past a row's IC elements
        const int rw = M >= 2048 ? 8 : (M >= 512 ? 4 : 1);   // table entries are fetched once per workgroup: several rows each
        const int nc = ceil_div(chunks, 256);
        auto kern = nc <= 1 ? gather_rows_reg_kernel<1> : (nc <= 2 ? gather_rows_reg_kernel<2> : gather_rows_reg_kernel<4>);
        kern<<<ceil_div(M, rw), 256, 2 * row_bytes, s>>>((const unsigned short*)X, (int)M, ldx, perm, ic, chunks, (unsigned short*)Xs, ldo, rw);
        return hipGetLastError();
    }
    if (row_bytes <= ROW_LDS_MAX && (ldx & 7) == 0 && ((uintptr_t)X & 15) == 0) {
        const int rw = rows_per_wg(M);
        gather_rows_kernel<<<ceil_div(M, rw), 256, row_bytes, s>>>((const unsigned short*)X, (int)M, ldx, perm, ic, chunks,
                                                                   (unsigned short*)Xs, ldo, rw);
        return hipGetLastError();
    }
    const int64_t n = M * chunks;
    gather_cols_kernel<<<ceil_div(n, 256), 256, 0, s>>>((const unsigned short*)X, (int)M, ldx, perm, ic, chunks,
                                                       (unsigned short*)Xs, ldo);
    return hipGetLastError();
}

hipError_t scatter_cols(const __half* Ds, int64_t M, const int* perm, int ic, __half* dX, int64_t lddx, hipStream_t s) {
    const int chunks = (ic + 7) / 8;
    const int row_bytes = chunks * 16;
    if (chunks <= 1024 && (lddx & 7) == 0 && ((uintptr_t)dX & 15) == 0) {
        const int rw = M >= 2048 ? 8 : (M >= 512 ? 4 : 1);
        const int nc = ceil_div(chunks, 256);
        auto kern = nc <= 1 ? scatter_rows_reg_kernel<1> : (nc <= 2 ? scatter_rows_reg_kernel<2> : scatter_rows_reg_kernel<4>);
        kern<<<ceil_div(M, rw), 256, 2 * row_bytes, s>>>((const unsigned short*)Ds, (int)M, (int64_t)chunks * 8, perm, ic, chunks,
                                                        (unsigned short*)dX, lddx, rw);
        return hipGetLastError();
    }
    if (row_bytes <= ROW_LDS_MAX && (lddx & 7) == 0 && ((uintptr_t)dX & 15) == 0) {
        const int rw = rows_per_wg(M);
        scatter_rows_kernel<<<ceil_div(M, rw), 256, row_bytes, s>>>((const unsigned short*)Ds, (int)M, (int64_t)chunks * 8, perm, ic,
                                                                    chunks, (unsigned short*)dX, lddx, rw);
        return hipGetLastError();
    }
    const int64_t n = M * chunks;
    scatter_cols_kernel<<<ceil_div(n, 256), 256, 0, s>>>((const unsigned short*)Ds, (int)M, (int64_t)chunks * 8, perm, ic, chunks,
                                                        (unsigned short*)dX, lddx);
    return hipGetLastError();
}

}  // namespace qeft
