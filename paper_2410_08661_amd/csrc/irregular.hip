// Weak columns at arbitrary input channels (paper Sec. 3.2, last paragraph; Limitations): the
// attention output projection cannot be reordered offline, so its stored form keeps the
// non-weak channels in ascending order followed by the weak block, and the activations are
// brought into that order on the fly.  Here that is a gather of X (and a scatter of dX)
// through a caller-provided workspace, around the kernels of the reordered layer:
//     Xs[m][j] = X[m][perm[j]]          dX[m][perm[j]] = dXs[m][j]
// perm (int32 [IC], device) holds the original channel of every stored column.  Entries are
// clamped to [0, IC) so that a malformed table can give wrong numbers but no access outside
// the matrices.
#include "qeft_internal.h"

namespace qeft {
namespace {

typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef int i4 __attribute__((ext_vector_type(4)));

// One thread per 8 stored columns of one row: two 16-byte reads of the table, eight 2-byte
// reads of X (scattered over the row, which stays in L2 / the last-level cache), one 16-byte store.
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

}  // namespace

size_t irregular_workspace(int ic, int64_t M) { return (size_t)M * (size_t)((ic + 7) / 8 * 8) * sizeof(__half); }

hipError_t gather_cols(const __half* X, int64_t M, int64_t ldx, const int* perm, int ic, __half* Xs, hipStream_t s) {
    const int chunks = (ic + 7) / 8;
    const int64_t n = M * chunks;
    gather_cols_kernel<<<ceil_div(n, 256), 256, 0, s>>>((const unsigned short*)X, (int)M, ldx, perm, ic, chunks,
                                                       (unsigned short*)Xs, (int64_t)chunks * 8);
    return hipGetLastError();
}

hipError_t scatter_cols(const __half* Ds, int64_t M, const int* perm, int ic, __half* dX, int64_t lddx, hipStream_t s) {
    const int chunks = (ic + 7) / 8;
    const int64_t n = M * chunks;
    scatter_cols_kernel<<<ceil_div(n, 256), 256, 0, s>>>((const unsigned short*)Ds, (int)M, (int64_t)chunks * 8, perm, ic, chunks,
                                                        (unsigned short*)dX, lddx);
    return hipGetLastError();
}

}  // namespace qeft
