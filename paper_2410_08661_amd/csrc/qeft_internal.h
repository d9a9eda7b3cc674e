// Internal declarations shared by the translation units of libqeft (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "qeft.h"

namespace qeft {

// Everything a kernel needs to know about one stored layer (see qeft.h for the format).
struct Layer {
    int oc, ic, k, bits, g;
    int dense;     // 1: dense 3-bit layout (a row's codes as one bit string), 0: whole codes per word
    int kq;        // ic - k
    int ng;        // groups per row
    int gs;        // row pitch of scales / zeros in elements (ng rounded up to a multiple of 8)
    int words;     // used words per row
    int stride;    // words per row incl. padding (multiple of 4)
    const uint32_t* qweight;
    const __half* scales;
    const __half* zeros;
    const __half* weak;
};

inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// Code of column j of a row of packed words, either layout (the plain definition: conversion and fallback kernels).
__device__ __forceinline__ uint32_t code_at(const Layer& L, const uint32_t* __restrict__ row, int j) {
    if (L.dense) {
        const int bit = 3 * j, w0 = bit >> 5, sh = bit & 31;
        uint32_t v = row[w0] >> sh;
        if (sh > 29) v |= row[w0 + 1] << (32 - sh);   // the code straddles two words (never the row's last one)
        return v & 7u;
    }
    const int per = (L.bits == 4) ? 8 : 10;
    return (row[j / per] >> (L.bits * (j % per))) & ((1u << L.bits) - 1u);
}

// ---- generic kernels: any shape, bits and alignment; plain loops (generic.hip) ------
hipError_t fwd_generic(const Layer& L, const __half* X, int64_t M, int64_t ldx, __half* Y, int64_t ldy, hipStream_t s);
hipError_t bwd_dx_generic(const Layer& L, const __half* dY, int64_t M, int64_t lddy, __half* dX, int64_t lddx, hipStream_t s);
hipError_t weak_grad_generic(int oc, int k, const __half* dY, int64_t M, int64_t lddy, const __half* Xw, int64_t ldxw,
                             void* dW, int out_f32, int accumulate, hipStream_t s);

// ---- weak columns at arbitrary channels: gather / scatter through a workspace (irregular.hip) ----
size_t irregular_workspace(int ic, int64_t M);   // [M][IC rounded up to 8] fp16
hipError_t gather_cols(const __half* X, int64_t M, int64_t ldx, const int* perm, int ic, __half* Xs, int64_t ldo, hipStream_t s);
hipError_t scatter_cols(const __half* Ds, int64_t M, const int* perm, int ic, __half* dX, int64_t lddx, hipStream_t s);

// ---- global weak-column selection and offline reordering (reorder.hip) --------------------------
size_t sens_workspace(int d, int64_t tokens);
hipError_t sensitivity(const __half* X, int64_t tokens, int64_t ldx, int d, int n_batch, float* out, float* ws, hipStream_t s);
hipError_t topk_vote(const float* v, int d, int k, int* idx_out, float* s_global, hipStream_t s);
hipError_t weak_order(const int* idx, int k, int d, int* perm, hipStream_t s);
hipError_t gather_rows16(const __half* W, int64_t ldw, const int* perm, int rows, int src_rows, int cols, __half* out, int64_t ldo,
                         hipStream_t s);

hipError_t merge_weak(const __half* tuned, const __half* base, int64_t oc, int k, const int* idx, int target_cols,
                      __half* target, int64_t ldt, hipStream_t s);

// ---- format conversion (pack.hip) ----------------------------------------------------
hipError_t pack_rtn(const Layer& L, const __half* W, int64_t ldw, uint32_t* qweight, __half* scales, __half* zeros,
                    __half* weak, hipStream_t s);
bool pack_search_supported(const Layer& L, int64_t ldw, const void* W);
hipError_t pack_search(const Layer& L, const __half* W, int64_t ldw, int n_grid, float step, uint32_t* qweight,
                       __half* scales, __half* zeros, __half* weak, hipStream_t s);
hipError_t pack_codes(const Layer& L, const uint8_t* codes, const __half* scales_in, const __half* zeros_in,
                      const __half* weak_in, uint32_t* qweight, __half* scales, __half* zeros, __half* weak, hipStream_t s);
hipError_t unpack(const Layer& L, uint8_t* codes, __half* scales, __half* zeros, __half* weak, hipStream_t s);
// The whole mixed weight as fp16 [OC][IC] (IC a multiple of 8): s (q - z) rounded once, then the weak block.
hipError_t dequantize_fp16(const Layer& L, __half* out, hipStream_t s);

// ---- decode path: fused dequant matrix-vector product for M <= 16 (gemv.hip) -------------
bool gemv_supported(const Layer& L, int64_t M, int64_t ldx);
hipError_t gemv_fwd(const Layer& L, const __half* X, int64_t M, int64_t ldx, __half* Y, int64_t ldy, hipStream_t s);
// Several layers that share the input (same IC, k, bits and group size; any OC each) in one
// launch of the small-M kernel: its row tiles are those of layer 0, then layer 1, ...
constexpr int MAX_GROUP = 4;
struct GroupTail {            // layers 1 .. 3 of a group (layer 0 travels as the kernel's Layer)
    const uint32_t* qweight[MAX_GROUP - 1];
    const __half* scales[MAX_GROUP - 1];
    const __half* zeros[MAX_GROUP - 1];
    const __half* weak[MAX_GROUP - 1];
    __half* Y[MAX_GROUP - 1];
    int64_t ldy[MAX_GROUP - 1];
    int oc[MAX_GROUP - 1];
    int tile_begin[MAX_GROUP - 1];   // first 16-row tile of the layer; INT_MAX when absent
};
// Decode with the activations in original channel order, gathered through perm inside the kernel
// (weak columns at arbitrary channels); *handled = false when the shape does not fit that kernel.
hipError_t gemv_fwd_perm(const Layer& L, const int* perm, const __half* X, int64_t M, int64_t ldx, __half* Y, int64_t ldy,
                         hipStream_t s, bool* handled);
// *handled = false (and nothing launched) when the shapes do not fit the one-launch kernel
hipError_t gemv_fwd_group(const Layer* Ls, int n, const __half* X, int64_t M, int64_t ldx, __half* const* Y,
                          const int64_t* ldy, hipStream_t s, bool* handled);

// Decode at M = 1: rows per wavefront, activations in registers (gemv_dot.hip).  Ls[0 .. n) share the input;
// perm (or nullptr) gathers the activations from original channel order.  *handled = false: not this kernel's shape.
hipError_t gemv_dot_fwd(const Layer* Ls, int n, const int* perm, const __half* X, __half* const* Y, hipStream_t s, bool* handled);

// ---- prefill / fine-tune path: MFMA GEMMs (gemm.hip) ---------------------------------------
bool gemm_fwd_supported(const Layer& L, int64_t M);
// ws: optional device workspace of gemm_fwd_split_workspace() bytes (16-byte aligned); with it, launches of few tiles, or with a
// sparsely filled last round of tiles, split K (for dX: the weight rows) of those tiles
hipError_t gemm_fwd(const Layer& L, const __half* X, int64_t M, int64_t ldx, __half* Y, int64_t ldy, void* ws, hipStream_t s);
size_t gemm_fwd_split_workspace(const Layer& L, int64_t M);
bool gemm_dx_supported(const Layer& L, int64_t M);
hipError_t gemm_dx(const Layer& L, const __half* dY, int64_t M, int64_t lddy, __half* dX, int64_t lddx, void* ws, hipStream_t s);
size_t gemm_dx_split_workspace(const Layer& L, int64_t M);
bool weak_grad_mfma_supported(int oc, int k, int64_t M);
size_t weak_grad_mfma_workspace(int oc, int k, int64_t M);
hipError_t weak_grad_mfma(int oc, int k, const __half* dY, int64_t M, int64_t lddy, const __half* Xw, int64_t ldxw,
                          void* dW, int out_f32, int accumulate, void* ws, hipStream_t s);

// input gradient and weak-block gradient of one layer in one launch (ws: the weak gradient's workspace)
bool gemm_dx_dw_supported(const Layer& L, int64_t M);
hipError_t gemm_dx_dw(const Layer& L, const __half* dY, int64_t M, int64_t lddy, __half* dX, int64_t lddx, const __half* Xw,
                      int64_t ldxw, void* dW, int out_f32, int accumulate, void* ws, hipStream_t s);

}  // namespace qeft
