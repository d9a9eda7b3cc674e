// Global weak-column selection and offline reordering (paper Sec. 3.2, App. B): the one-time
// preparation that makes every layer's weak columns the same contiguous block.
//   sensitivity   s_j = (2 / n_batch) sum_t X[t][j]^2, the diagonal of the layer input's Hessian
//   vote          a layer's k most sensitive channels add s_j / mean(s) to the global score
//   top-k         the k channels with the largest global score (ties: lower index first)
//   order         the permutation that moves them to the end (non-weak channels ascending first)
//   reorder       a matrix's columns or rows taken in that order
// None of this is on the inference or fine-tuning path; the kernels are plain and bandwidth-bound
// where it matters (sensitivity reads the activations once with 16-byte loads).
#include "qeft_internal.h"

namespace qeft {
namespace {

typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));

// Workgroup (32 column octets x 8 token lanes): partial sums of squares of 256 columns over the
// tokens split, split + splits, ...; combined through LDS in a fixed order, one fp32 slab per split.
__global__ __launch_bounds__(256) void sens_partial_kernel(const __half* __restrict__ X, int64_t tokens, int64_t ldx, int d,
                                                           int chunks, int splits, float* __restrict__ part) {
    __shared__ float red[8][32][8];
    const int oct = threadIdx.x & 31, tl = threadIdx.x >> 5;
    const int cb = blockIdx.x % chunks, split = blockIdx.x / chunks;
    const int col = 256 * cb + 8 * oct;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (col < d) {   // d % 8 == 0: whole octets
        for (int64_t t = (int64_t)split * 8 + tl; t < tokens; t += (int64_t)splits * 8) {
            const h8 h = __builtin_bit_cast(h8, *reinterpret_cast<const u4*>(X + (size_t)t * ldx + col));
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = fmaf((float)h[e], (float)h[e], acc[e]);
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[tl][oct][e] = acc[e];
    __syncthreads();
    if (tl == 0 && col < d) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float s = red[0][oct][e];
            for (int l = 1; l < 8; ++l) s += red[l][oct][e];
            part[(size_t)split * d + col + e] = s;
        }
    }
}

__global__ __launch_bounds__(256) void sens_finish_kernel(const float* __restrict__ part, int splits, int d, float scale,
                                                          float* __restrict__ out) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= d) return;
    float s = 0.f;
    for (int p = 0; p < splits; ++p) s += part[(size_t)p * d + j];
    out[j] = s * scale;
}

// rank of every entry (number of entries that come before it: larger, or equal with a lower
// index); the first k write their index at their rank and, when a global score is given, add
// their value relative to the mean.  Every workgroup sums all of v itself (d is a few tens of
// thousands at most) so that one launch suffices.
__global__ __launch_bounds__(256) void topk_vote_kernel(const float* __restrict__ v, int d, int k, int* __restrict__ idx_out,
                                                        float* __restrict__ s_global) {
    __shared__ float tile[256];
    const int j = blockIdx.x * 256 + threadIdx.x;
    const float mine = j < d ? v[j] : 0.f;
    int rank = 0;
    float total = 0.f;
    for (int base = 0; base < d; base += 256) {
        const int i = base + threadIdx.x;
        tile[threadIdx.x] = i < d ? v[i] : -__builtin_inff();
        __syncthreads();
        const int n = min(256, d - base);
        for (int t = 0; t < n; ++t) {
            const float o = tile[t];
            rank += (o > mine) || (o == mine && base + t < j);
        }
        if (s_global) {   // fixed order: tile by tile, within a tile left to right (the same in every workgroup)
            float ts = 0.f;
            for (int t = 0; t < n; ++t) ts += tile[t];
            total += ts;
        }
        __syncthreads();
    }
    if (j < d && rank < k) {
        idx_out[rank] = j;
        if (s_global) s_global[j] += mine / (total / (float)d);
    }
}

// perm: the non-weak channels in ascending order, then the weak ones as listed
__global__ __launch_bounds__(256) void weak_order_kernel(const int* __restrict__ idx, int k, int d, int* __restrict__ perm) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= d) return;
    int below = 0;
    bool weak = false;
    for (int c = 0; c < k; ++c) {
        const int w = idx[c];
        below += w < j;
        weak |= w == j;
    }
    if (!weak) perm[j - below] = j;
    if (j < k) perm[d - k + j] = min(max(idx[j], 0), d - 1);
}

// out[r][:] = W[perm[r]][:]  (16-byte pieces; cols % 8 == 0)
__global__ __launch_bounds__(256) void gather_rows16_kernel(const __half* __restrict__ W, int64_t ldw, const int* __restrict__ perm,
                                                            int rows, int src_rows, int chunks, __half* __restrict__ out, int64_t ldo) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= (int64_t)rows * chunks) return;
    const int r = (int)(t / chunks), c = (int)(t % chunks);
    const int src = min(max(perm[r], 0), src_rows - 1);
    *reinterpret_cast<u4*>(out + (size_t)r * ldo + 8 * c) = *reinterpret_cast<const u4*>(W + (size_t)src * ldw + 8 * c);
}

// target[o][idx[c]] (or target[o][c] without idx) += tuned[o][c] - base[o][c]: the difference is exact
// in fp32, the sum is one fp32 addition, the result one rounding to fp16
__global__ __launch_bounds__(256) void merge_weak_kernel(const __half* __restrict__ tuned, const __half* __restrict__ base,
                                                         int64_t oc, int k, const int* __restrict__ idx, int target_cols,
                                                         __half* __restrict__ target, int64_t ldt) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= oc * k) return;
    const int64_t o = t / k;
    const int c = (int)(t % k);
    const int col = idx ? min(max(idx[c], 0), target_cols - 1) : c;
    const float delta = __fsub_rn(__half2float(tuned[t]), __half2float(base[t]));
    __half* p = target + (size_t)o * ldt + col;
    *p = __float2half_rn(__fadd_rn(__half2float(*p), delta));
}

}  // namespace

hipError_t merge_weak(const __half* tuned, const __half* base, int64_t oc, int k, const int* idx, int target_cols,
                      __half* target, int64_t ldt, hipStream_t s) {
    merge_weak_kernel<<<ceil_div(oc * k, 256), 256, 0, s>>>(tuned, base, oc, k, idx, target_cols, target, ldt);
    return hipGetLastError();
}

int sens_splits(int d, int64_t tokens) {
    const int chunks = ceil_div(d, 256);
    int64_t s = ceil_div(2048, chunks);
    const int64_t cap = (tokens + 7) / 8;
    if (s > cap) s = cap;
    return (int)(s < 1 ? 1 : s);
}

size_t sens_workspace(int d, int64_t tokens) { return (size_t)sens_splits(d, tokens) * d * sizeof(float); }

hipError_t sensitivity(const __half* X, int64_t tokens, int64_t ldx, int d, int n_batch, float* out, float* ws, hipStream_t s) {
    const int chunks = ceil_div(d, 256), splits = sens_splits(d, tokens);
    sens_partial_kernel<<<chunks * splits, 256, 0, s>>>(X, tokens, ldx, d, chunks, splits, ws);
    sens_finish_kernel<<<ceil_div(d, 256), 256, 0, s>>>(ws, splits, d, 2.f / (float)n_batch, out);
    return hipGetLastError();
}

hipError_t topk_vote(const float* v, int d, int k, int* idx_out, float* s_global, hipStream_t s) {
    topk_vote_kernel<<<ceil_div(d, 256), 256, 0, s>>>(v, d, k, idx_out, s_global);
    return hipGetLastError();
}

hipError_t weak_order(const int* idx, int k, int d, int* perm, hipStream_t s) {
    weak_order_kernel<<<ceil_div(d, 256), 256, 0, s>>>(idx, k, d, perm);
    return hipGetLastError();
}

hipError_t gather_rows16(const __half* W, int64_t ldw, const int* perm, int rows, int src_rows, int cols, __half* out, int64_t ldo,
                         hipStream_t s) {
    const int chunks = cols / 8;
    gather_rows16_kernel<<<ceil_div((int64_t)rows * chunks, 256), 256, 0, s>>>(W, ldw, perm, rows, src_rows, chunks, out, ldo);
    return hipGetLastError();
}

}  // namespace qeft
