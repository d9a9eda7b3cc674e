// The C ABI (include/qeft.h): argument checks, layout arithmetic and kernel dispatch.
// Every check runs on the host before anything is launched.
#include "qeft_internal.h"

using namespace qeft;

namespace {

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

int check_desc(const qeft_desc_t* d) {
    if (!d) return QEFT_ERR_NULL;
    if (d->bits != 3 && d->bits != 4) return QEFT_ERR_BITS;
    if (d->out_features <= 0 || d->in_features <= 0 || d->group_size <= 0 || d->n_weak < 0 ||
        d->n_weak > d->in_features)
        return QEFT_ERR_SHAPE;
    if (d->out_features > QEFT_MAX_DIM || d->in_features > QEFT_MAX_DIM || d->group_size > QEFT_MAX_DIM) return QEFT_ERR_SHAPE;
    if (d->layout != QEFT_LAYOUT_CANONICAL && !(d->layout == QEFT_LAYOUT_DENSE3 && d->bits == 3)) return QEFT_ERR_UNSUPPORTED;
    return QEFT_OK;
}

void fill_layout(const qeft_desc_t* d, qeft_layout_t* o) {
    const int64_t per = (d->bits == 4) ? 8 : 10;
    o->kq = (int64_t)d->in_features - d->n_weak;
    o->n_groups = (o->kq + d->group_size - 1) / d->group_size;
    o->words_per_row = d->layout == QEFT_LAYOUT_DENSE3 ? (3 * o->kq + 31) / 32 : (o->kq + per - 1) / per;
    o->row_stride_words = (o->words_per_row + 15) / 16 * 16;
    o->qweight_bytes = (size_t)d->out_features * (size_t)o->row_stride_words * 4u;
    o->group_stride = (o->n_groups + 7) / 8 * 8;
    o->scales_bytes = (size_t)d->out_features * (size_t)o->group_stride * 2u;
    o->zeros_bytes = o->scales_bytes;
    o->weak_bytes = (size_t)d->out_features * (size_t)d->n_weak * 2u;
}

// Checks the four component pointers and fills the kernel-side description.
int make_layer(const qeft_desc_t* d, const qeft_weight_t* w, Layer* L) {
    int st = check_desc(d);
    if (st != QEFT_OK) return st;
    if (!w) return QEFT_ERR_NULL;
    qeft_layout_t lay;
    fill_layout(d, &lay);
    if (lay.kq > 0 && (!w->qweight || !w->scales || !w->zeros)) return QEFT_ERR_NULL;
    if (d->n_weak > 0 && !w->weak) return QEFT_ERR_NULL;
    if (lay.kq > 0 && (!aligned16(w->qweight) || !aligned16(w->scales) || !aligned16(w->zeros))) return QEFT_ERR_ALIGN;
    if (d->n_weak > 0 && !aligned16(w->weak)) return QEFT_ERR_ALIGN;
    L->oc = d->out_features;
    L->ic = d->in_features;
    L->k = d->n_weak;
    L->bits = d->bits;
    L->g = d->group_size;
    L->dense = d->layout == QEFT_LAYOUT_DENSE3;
    L->kq = (int)lay.kq;
    L->ng = (int)lay.n_groups;
    L->gs = (int)lay.group_stride;
    L->words = (int)lay.words_per_row;
    L->stride = (int)lay.row_stride_words;
    L->qweight = (const uint32_t*)w->qweight;
    L->scales = (const __half*)w->scales;
    L->zeros = (const __half*)w->zeros;
    L->weak = (const __half*)w->weak;
    return QEFT_OK;
}

int check_matrix(const void* p, int64_t M, int64_t ld, int64_t width) {
    if (M < 0 || M > QEFT_MAX_DIM) return QEFT_ERR_SHAPE;
    if (M == 0) return QEFT_OK;
    if (!p) return QEFT_ERR_NULL;
    if (ld < width) return QEFT_ERR_SHAPE;
    if (!aligned16(p) || (ld & 7) != 0) return QEFT_ERR_ALIGN;
    return QEFT_OK;
}

inline int hip_status(hipError_t e) { return e == hipSuccess ? QEFT_OK : QEFT_ERR_HIP; }

// Between the matrix-vector kernels (16 tokens per pass, the whole layer streamed per pass) and the tiled GEMM
// (256-token tiles: with few tokens only OC / 256 workgroups exist, a fraction of the 256 CUs, and each walks the
// whole K range) lies a range of token counts where repeated passes are faster.  Both are modelled from
// measurements on the Llama-2 shapes: a pass takes about 4.5 us + stored bytes / 4 TB/s + 0.85 us per 1000
// input channels, a GEMM ceil(tiles / 256) x stages x 1.15 us + 8 us; passes are taken when the model favours them by 10 %.
// (4096 x 4096: up to 96 tokens, 62 us against 75; 28672 x 8192: up to 32, 102 us against 152.)  Layers under
// 4 MB keep the GEMM: either way takes microseconds there.
bool passes_beat_gemm(const Layer& L, int64_t M) {
    if (M <= 16 || M > 256 || L.bits != 4) return false;
    const double bytes = (double)L.oc * ((double)L.stride * 4.0 + (double)L.gs * 4.0 + (double)L.k * 2.0);
    if (bytes < 4.0e6) return false;
    const double passes = (double)((M + 15) / 16), t_pass = 4.5 + bytes / 4.0e6 + 0.85e-3 * (double)L.ic;
    const double tiles = (double)((L.oc + 255) / 256), stages = (double)((L.kq + 63) / 64 + (L.k + 63) / 64);
    const double t_gemm = (double)((int64_t)(tiles + 255.0) / 256) * stages * 1.15 + 8.0;
    return passes * t_pass < 0.9 * t_gemm;
}

// 3-bit layers at GEMM sizes: the tiled kernels convert 4-bit codes only, so the layer is dequantized once
// into a caller-provided fp16 [OC][IC] workspace and multiplied as a layer whose columns are all weak
// (the paper's own training path: dequantize, then a dense product; Sec. 4.3 / App. A.2).
bool dense_copy_applies(const Layer& L, int64_t M) {
    return L.bits == 3 && L.kq > 0 && M > 16 && (L.ic % 8) == 0 && (L.oc % 8) == 0;
}
size_t dense_copy_bytes(const Layer& L) { return (size_t)L.oc * (size_t)L.ic * sizeof(__half); }
Layer dense_copy_layer(const Layer& L, const void* ws) {
    Layer D = L;
    D.bits = 4;
    D.dense = 0;
    D.g = 128;
    D.kq = 0;
    D.ng = D.gs = D.words = D.stride = 0;
    D.k = L.ic;
    D.qweight = nullptr;
    D.scales = D.zeros = nullptr;
    D.weak = (const __half*)ws;
    return D;
}

}  // namespace

extern "C" {

int qeft_layout(const qeft_desc_t* desc, qeft_layout_t* out) {
    int st = check_desc(desc);
    if (st != QEFT_OK) return st;
    if (!out) return QEFT_ERR_NULL;
    fill_layout(desc, out);
    return QEFT_OK;
}

int qeft_pack(const qeft_desc_t* desc, const void* W, int64_t ldw, const qeft_weight_t* out, void* stream) {
    Layer L;
    int st = make_layer(desc, out, &L);
    if (st != QEFT_OK) return st;
    st = check_matrix(W, L.oc, ldw, L.ic);
    if (st != QEFT_OK) return st;
    return hip_status(pack_rtn(L, (const __half*)W, ldw, (uint32_t*)out->qweight, (__half*)out->scales,
                               (__half*)out->zeros, (__half*)out->weak, (hipStream_t)stream));
}

int qeft_pack_search(const qeft_desc_t* desc, const void* W, int64_t ldw, int n_grid, float shrink_step,
                     const qeft_weight_t* out, void* stream) {
    Layer L;
    int st = make_layer(desc, out, &L);
    if (st != QEFT_OK) return st;
    st = check_matrix(W, L.oc, ldw, L.ic);
    if (st != QEFT_OK) return st;
    if (n_grid < 1 || !(shrink_step >= 0.f) || !((float)(n_grid - 1) * shrink_step < 1.f)) return QEFT_ERR_SHAPE;
    if (!pack_search_supported(L, ldw, W)) return QEFT_ERR_UNSUPPORTED;
    return hip_status(pack_search(L, (const __half*)W, ldw, n_grid, shrink_step, (uint32_t*)out->qweight,
                                  (__half*)out->scales, (__half*)out->zeros, (__half*)out->weak, (hipStream_t)stream));
}

int qeft_pack_codes(const qeft_desc_t* desc, const uint8_t* codes, const void* scales, const void* zeros,
                    const void* weak, const qeft_weight_t* out, void* stream) {
    Layer L;
    int st = make_layer(desc, out, &L);
    if (st != QEFT_OK) return st;
    if (L.kq > 0 && (!codes || !scales || !zeros)) return QEFT_ERR_NULL;
    if (L.k > 0 && !weak) return QEFT_ERR_NULL;
    return hip_status(pack_codes(L, codes, (const __half*)scales, (const __half*)zeros, (const __half*)weak,
                                 (uint32_t*)out->qweight, (__half*)out->scales, (__half*)out->zeros,
                                 (__half*)out->weak, (hipStream_t)stream));
}

int qeft_unpack(const qeft_desc_t* desc, const qeft_weight_t* w, uint8_t* codes, void* scales, void* zeros,
                void* weak, void* stream) {
    Layer L;
    int st = make_layer(desc, w, &L);
    if (st != QEFT_OK) return st;
    return hip_status(unpack(L, codes, (__half*)scales, (__half*)zeros, (__half*)weak, (hipStream_t)stream));
}

size_t qeft_workspace_bytes(const qeft_desc_t* desc, int op, int64_t M) {
    if (check_desc(desc) != QEFT_OK || M <= 0 || M > QEFT_MAX_DIM) return 0;
    if (op == QEFT_OP_WEAK_GRAD && weak_grad_mfma_supported(desc->out_features, desc->n_weak, M))
        return weak_grad_mfma_workspace(desc->out_features, desc->n_weak, M);
    if (op == QEFT_OP_BWD) {   // the two steps use the workspace one after the other
        const size_t a = qeft_workspace_bytes(desc, QEFT_OP_WEAK_GRAD, M), b = qeft_workspace_bytes(desc, QEFT_OP_BWD_DX, M);
        return a > b ? a : b;
    }
    if (op == QEFT_OP_FWD_IRREGULAR || op == QEFT_OP_BWD_DX_IRREGULAR) return irregular_workspace(desc->in_features, M);
    if (op == QEFT_OP_FWD || op == QEFT_OP_BWD_DX) {
        Layer L = {};
        L.bits = desc->bits;
        L.oc = desc->out_features;
        L.ic = desc->in_features;
        L.k = desc->n_weak;
        L.g = desc->group_size;
        L.kq = desc->in_features - desc->n_weak;
        if (dense_copy_applies(L, M)) {
            // the fp16 copy; behind it the partial tiles of a split of the copy's columns (forward) or rows (input gradient)
            const Layer D = dense_copy_layer(L, nullptr);
            if (op == QEFT_OP_FWD) return dense_copy_bytes(L) + (gemm_fwd_supported(D, M) ? gemm_fwd_split_workspace(D, M) : 0);
            return dense_copy_bytes(L) + (gemm_dx_supported(D, M) ? gemm_dx_split_workspace(D, M) : 0);
        }
        if (op == QEFT_OP_FWD && M > 16 && gemm_fwd_supported(L, M)) return gemm_fwd_split_workspace(L, M);
        if (op == QEFT_OP_BWD_DX && gemm_dx_supported(L, M)) return gemm_dx_split_workspace(L, M);
    }
    return 0;
}

int qeft_linear_fwd(const qeft_desc_t* desc, const qeft_weight_t* w, const void* X, int64_t M, int64_t ldx,
                    void* Y, int64_t ldy, void* ws, size_t ws_bytes, void* stream) {
    Layer L;
    int st = make_layer(desc, w, &L);
    if (st != QEFT_OK) return st;
    st = check_matrix(X, M, ldx, L.ic);
    if (st != QEFT_OK) return st;
    st = check_matrix(Y, M, ldy, L.oc);
    if (st != QEFT_OK) return st;
    if (M == 0) return QEFT_OK;
    hipStream_t s = (hipStream_t)stream;
    const __half* x = (const __half*)X;
    __half* y = (__half*)Y;
    if (M > 16 && gemm_fwd_supported(L, M)) {
        // optional workspace: K-split partial tiles for launches of few tiles
        const size_t need = ws ? gemm_fwd_split_workspace(L, M) : 0;
        if (need > 0) {
            if (!aligned16(ws)) return QEFT_ERR_ALIGN;
            if (ws_bytes < need) return QEFT_ERR_WORKSPACE;
        }
        if (need > 0 ? M >= 48 : !(passes_beat_gemm(L, M) && gemv_supported(L, 16, ldx)))
            return hip_status(gemm_fwd(L, x, M, ldx, y, ldy, need > 0 ? ws : nullptr, s));
    }
    if (ws && dense_copy_applies(L, M)) {
        if (!aligned16(ws)) return QEFT_ERR_ALIGN;
        if (ws_bytes < dense_copy_bytes(L)) return QEFT_ERR_WORKSPACE;
        const Layer D = dense_copy_layer(L, ws);
        if (gemm_fwd_supported(D, M)) {
            hipError_t e = dequantize_fp16(L, (__half*)ws, s);
            if (e != hipSuccess) return QEFT_ERR_HIP;
            // what the caller gave beyond the copy serves a split of its columns (all of it or nothing)
            const size_t need = gemm_fwd_split_workspace(D, M);
            void* split_ws = (need > 0 && ws_bytes >= dense_copy_bytes(L) + need) ? (char*)ws + dense_copy_bytes(L) : nullptr;
            return hip_status(gemm_fwd(D, x, M, ldx, y, ldy, split_ws, s));
        }
    }
    if (gemv_supported(L, M, ldx)) {
        // the matrix-vector kernel takes up to 16 rows per pass
        for (int64_t m0 = 0; m0 < M; m0 += 16) {
            const int64_t mm = (M - m0 < 16) ? (M - m0) : 16;
            hipError_t e = gemv_fwd(L, x + m0 * ldx, mm, ldx, y + m0 * ldy, ldy, s);
            if (e != hipSuccess) return QEFT_ERR_HIP;
        }
        return QEFT_OK;
    }
    return hip_status(fwd_generic(L, x, M, ldx, y, ldy, s));
}

int qeft_linear_fwd_group(int n, const qeft_desc_t* descs, const qeft_weight_t* w, const void* X, int64_t M,
                          int64_t ldx, void* const* Y, const int64_t* ldy, void* stream) {
    if (n < 1 || n > QEFT_MAX_GROUP) return QEFT_ERR_SHAPE;
    if (!descs || !w || !Y || !ldy) return QEFT_ERR_NULL;
    Layer Ls[QEFT_MAX_GROUP];
    for (int i = 0; i < n; ++i) {
        int st = make_layer(&descs[i], &w[i], &Ls[i]);
        if (st != QEFT_OK) return st;
        if (Ls[i].ic != Ls[0].ic || Ls[i].k != Ls[0].k || Ls[i].bits != Ls[0].bits || Ls[i].g != Ls[0].g || Ls[i].dense != Ls[0].dense) return QEFT_ERR_SHAPE;
        st = check_matrix(Y[i], M, ldy[i], Ls[i].oc);
        if (st != QEFT_OK) return st;
    }
    int st = check_matrix(X, M, ldx, Ls[0].ic);
    if (st != QEFT_OK) return st;
    if (M == 0) return QEFT_OK;
    hipStream_t s = (hipStream_t)stream;
    if (n > 1 && M <= 16 && gemv_supported(Ls[0], M, ldx)) {
        __half* ys[QEFT_MAX_GROUP];
        for (int i = 0; i < n; ++i) ys[i] = (__half*)Y[i];
        bool handled = false;
        hipError_t e = gemv_fwd_group(Ls, n, (const __half*)X, M, ldx, ys, ldy, s, &handled);
        if (e != hipSuccess) return QEFT_ERR_HIP;
        if (handled) return QEFT_OK;
    }
    for (int i = 0; i < n; ++i) {
        st = qeft_linear_fwd(&descs[i], &w[i], X, M, ldx, Y[i], ldy[i], nullptr, 0, stream);
        if (st != QEFT_OK) return st;
    }
    return QEFT_OK;
}

int qeft_linear_bwd_dx(const qeft_desc_t* desc, const qeft_weight_t* w, const void* dY, int64_t M, int64_t lddy,
                       void* dX, int64_t lddx, void* ws, size_t ws_bytes, void* stream) {
    Layer L;
    int st = make_layer(desc, w, &L);
    if (st != QEFT_OK) return st;
    st = check_matrix(dY, M, lddy, L.oc);
    if (st != QEFT_OK) return st;
    st = check_matrix(dX, M, lddx, L.ic);
    if (st != QEFT_OK) return st;
    if (M == 0) return QEFT_OK;
    hipStream_t s = (hipStream_t)stream;
    if (gemm_dx_supported(L, M)) {
        const size_t need = ws ? gemm_dx_split_workspace(L, M) : 0;   // optional: partial tiles of a row split
        if (need > 0) {
            if (!aligned16(ws)) return QEFT_ERR_ALIGN;
            if (ws_bytes < need) return QEFT_ERR_WORKSPACE;
        }
        return hip_status(gemm_dx(L, (const __half*)dY, M, lddy, (__half*)dX, lddx, need > 0 ? ws : nullptr, s));
    }
    if (ws && dense_copy_applies(L, M)) {
        if (!aligned16(ws)) return QEFT_ERR_ALIGN;
        if (ws_bytes < dense_copy_bytes(L)) return QEFT_ERR_WORKSPACE;
        const Layer D = dense_copy_layer(L, ws);
        if (gemm_dx_supported(D, M)) {
            hipError_t e = dequantize_fp16(L, (__half*)ws, s);
            if (e != hipSuccess) return QEFT_ERR_HIP;
            // what the caller gave beyond the copy serves a row split of it (all of it or nothing)
            const size_t need = gemm_dx_split_workspace(D, M);
            void* split_ws = (need > 0 && ws_bytes >= dense_copy_bytes(L) + need) ? (char*)ws + dense_copy_bytes(L) : nullptr;
            return hip_status(gemm_dx(D, (const __half*)dY, M, lddy, (__half*)dX, lddx, split_ws, s));
        }
    }
    return hip_status(bwd_dx_generic(L, (const __half*)dY, M, lddy, (__half*)dX, lddx, s));
}

int qeft_linear_fwd_irregular(const qeft_desc_t* desc, const qeft_weight_t* w, const int32_t* perm, const void* X,
                              int64_t M, int64_t ldx, void* Y, int64_t ldy, void* ws, size_t ws_bytes, void* stream) {
    int st = check_desc(desc);
    if (st != QEFT_OK) return st;
    const int ic = desc->in_features;
    st = check_matrix(X, M, ldx, ic);
    if (st != QEFT_OK) return st;
    if (M == 0) return qeft_linear_fwd(desc, w, X, M, ldx, Y, ldy, nullptr, 0, stream);
    if (!perm) return QEFT_ERR_NULL;
    if (!aligned16(perm)) return QEFT_ERR_ALIGN;
    if (M <= 4) {   // decode: the gather happens inside the matrix-vector kernel, no workspace
        Layer L;
        st = make_layer(desc, w, &L);
        if (st != QEFT_OK) return st;
        st = check_matrix(Y, M, ldy, L.oc);
        if (st != QEFT_OK) return st;
        if (gemv_supported(L, M, ldx)) {
            bool handled = false;
            if (gemv_fwd_perm(L, perm, (const __half*)X, M, ldx, (__half*)Y, ldy, (hipStream_t)stream, &handled) != hipSuccess)
                return QEFT_ERR_HIP;
            if (handled) return QEFT_OK;
        }
    }
    const size_t need = irregular_workspace(ic, M);
    if (!ws || ws_bytes < need || !aligned16(ws)) return QEFT_ERR_WORKSPACE;
    // validate the product's arguments before the gather is launched (M = 0 launches nothing)
    st = qeft_linear_fwd(desc, w, ws, 0, (ic + 7) / 8 * 8, Y, ldy, nullptr, 0, stream);
    if (st != QEFT_OK) return st;
    st = check_matrix(Y, M, ldy, desc->out_features);
    if (st != QEFT_OK) return st;
    if (gather_cols((const __half*)X, M, ldx, perm, ic, (__half*)ws, (ic + 7) / 8 * 8, (hipStream_t)stream) != hipSuccess) return QEFT_ERR_HIP;
    return qeft_linear_fwd(desc, w, ws, M, (ic + 7) / 8 * 8, Y, ldy, nullptr, 0, stream);
}

int qeft_linear_bwd_dx_irregular(const qeft_desc_t* desc, const qeft_weight_t* w, const int32_t* perm, const void* dY,
                                 int64_t M, int64_t lddy, void* dX, int64_t lddx, void* ws, size_t ws_bytes,
                                 void* stream) {
    int st = check_desc(desc);
    if (st != QEFT_OK) return st;
    const int ic = desc->in_features;
    st = check_matrix(dX, M, lddx, ic);
    if (st != QEFT_OK) return st;
    if (M == 0) return qeft_linear_bwd_dx(desc, w, dY, M, lddy, dX, lddx, nullptr, 0, stream);
    if (!perm) return QEFT_ERR_NULL;
    if (!aligned16(perm)) return QEFT_ERR_ALIGN;
    const size_t need = irregular_workspace(ic, M);
    if (!ws || ws_bytes < need || !aligned16(ws)) return QEFT_ERR_WORKSPACE;
    st = qeft_linear_bwd_dx(desc, w, dY, M, lddy, ws, (ic + 7) / 8 * 8, nullptr, 0, stream);
    if (st != QEFT_OK) return st;
    return hip_status(scatter_cols((const __half*)ws, M, perm, ic, (__half*)dX, lddx, (hipStream_t)stream));
}

size_t qeft_sensitivity_workspace(int32_t d, int64_t tokens) {
    if (d <= 0 || tokens <= 0 || d > QEFT_MAX_DIM || tokens > ((int64_t)1 << 31)) return 0;
    return sens_workspace(d, tokens);
}

int qeft_sensitivity(const void* X, int64_t tokens, int64_t ldx, int32_t d, int32_t n_batch, float* out, void* ws,
                     size_t ws_bytes, void* stream) {
    if (d <= 0 || (d & 7) != 0 || tokens <= 0 || n_batch <= 0 || d > QEFT_MAX_DIM || tokens > ((int64_t)1 << 31)) return QEFT_ERR_SHAPE;
    int st = check_matrix(X, tokens, ldx, d);
    if (st != QEFT_OK) return st;
    if (!out) return QEFT_ERR_NULL;
    if (!ws || ws_bytes < sens_workspace(d, tokens) || !aligned16(ws)) return QEFT_ERR_WORKSPACE;
    return hip_status(sensitivity((const __half*)X, tokens, ldx, d, n_batch, out, (float*)ws, (hipStream_t)stream));
}

int qeft_vote(const float* s, int32_t d, int32_t k, int32_t* idx_out, float* s_global, void* stream) {
    if (d <= 0 || k < 0 || k > d) return QEFT_ERR_SHAPE;
    if (!s || (k > 0 && !idx_out)) return QEFT_ERR_NULL;
    if (k == 0) return QEFT_OK;
    return hip_status(topk_vote(s, d, k, idx_out, s_global, (hipStream_t)stream));
}

int qeft_weak_order(const int32_t* idx, int32_t k, int32_t d, int32_t* perm, void* stream) {
    if (d <= 0 || k < 0 || k > d) return QEFT_ERR_SHAPE;
    if (!perm || (k > 0 && !idx)) return QEFT_ERR_NULL;
    return hip_status(weak_order(idx, k, d, perm, (hipStream_t)stream));
}

int qeft_reorder(const void* A, int64_t rows, int64_t cols, int64_t lda, const int32_t* perm, int axis, void* out,
                 int64_t ldo, void* stream) {
    if (rows < 0 || cols < 0 || (axis != 0 && axis != 1)) return QEFT_ERR_SHAPE;
    if (rows == 0 || cols == 0) return QEFT_OK;
    int st = check_matrix(A, rows, lda, cols);
    if (st != QEFT_OK) return st;
    st = check_matrix(out, rows, ldo, cols);
    if (st != QEFT_OK) return st;
    if (!perm) return QEFT_ERR_NULL;
    if (A == out) return QEFT_ERR_SHAPE;   // not in place
    if (axis == 1) return hip_status(gather_cols((const __half*)A, rows, lda, perm, (int)cols, (__half*)out, ldo, (hipStream_t)stream));
    if ((cols & 7) != 0) return QEFT_ERR_UNSUPPORTED;
    return hip_status(gather_rows16((const __half*)A, lda, perm, (int)rows, (int)rows, (int)cols, (__half*)out, ldo, (hipStream_t)stream));
}

int qeft_merge_weak(const void* tuned, const void* base, int64_t out_features, int32_t k, const int32_t* idx, void* target,
                    int64_t ldt, int32_t target_cols, void* stream) {
    if (out_features < 0 || k < 0 || target_cols < k || ldt < target_cols) return QEFT_ERR_SHAPE;
    if (out_features == 0 || k == 0) return QEFT_OK;
    if (!tuned || !base || !target) return QEFT_ERR_NULL;
    return hip_status(merge_weak((const __half*)tuned, (const __half*)base, out_features, k, idx, target_cols, (__half*)target,
                                 ldt, (hipStream_t)stream));
}

int qeft_weak_grad(const qeft_desc_t* desc, const void* dY, int64_t M, int64_t lddy, const void* Xw, int64_t ldxw,
                   void* dW, int out_dtype, int accumulate, void* ws, size_t ws_bytes, void* stream) {
    int st = check_desc(desc);
    if (st != QEFT_OK) return st;
    if (out_dtype != QEFT_DTYPE_F16 && out_dtype != QEFT_DTYPE_F32) return QEFT_ERR_UNSUPPORTED;
    const int oc = desc->out_features, k = desc->n_weak;
    st = check_matrix(dY, M, lddy, oc);
    if (st != QEFT_OK) return st;
    if (k == 0 || M == 0) return (M < 0) ? QEFT_ERR_SHAPE : QEFT_OK;
    st = check_matrix(Xw, M, ldxw, k);
    if (st != QEFT_OK) return st;
    if (!dW) return QEFT_ERR_NULL;
    if (!aligned16(dW)) return QEFT_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    if (weak_grad_mfma_supported(oc, k, M)) {
        const size_t need = weak_grad_mfma_workspace(oc, k, M);
        if (need > 0 && (!ws || ws_bytes < need || !aligned16(ws))) return QEFT_ERR_WORKSPACE;
        return hip_status(weak_grad_mfma(oc, k, (const __half*)dY, M, lddy, (const __half*)Xw, ldxw, dW,
                                         out_dtype == QEFT_DTYPE_F32, accumulate != 0, ws, s));
    }
    return hip_status(weak_grad_generic(oc, k, (const __half*)dY, M, lddy, (const __half*)Xw, ldxw, dW,
                                        out_dtype == QEFT_DTYPE_F32, accumulate != 0, s));
}

int qeft_linear_bwd(const qeft_desc_t* desc, const qeft_weight_t* w, const void* dY, int64_t M, int64_t lddy, void* dX,
                    int64_t lddx, const void* Xw, int64_t ldxw, void* dW, int out_dtype, int accumulate, void* ws,
                    size_t ws_bytes, void* stream) {
    Layer L;
    int st = make_layer(desc, w, &L);
    if (st != QEFT_OK) return st;
    if (out_dtype != QEFT_DTYPE_F16 && out_dtype != QEFT_DTYPE_F32) return QEFT_ERR_UNSUPPORTED;
    st = check_matrix(dY, M, lddy, L.oc);
    if (st != QEFT_OK) return st;
    st = check_matrix(dX, M, lddx, L.ic);
    if (st != QEFT_OK) return st;
    if (M == 0) return QEFT_OK;
    if (L.k == 0) return qeft_linear_bwd_dx(desc, w, dY, M, lddy, dX, lddx, nullptr, 0, stream);
    st = check_matrix(Xw, M, ldxw, L.k);
    if (st != QEFT_OK) return st;
    if (!dW) return QEFT_ERR_NULL;
    if (!aligned16(dW)) return QEFT_ERR_ALIGN;
    // the weak gradient's workspace is required whichever way the two steps run; checked before any launch
    const size_t need_dw = weak_grad_mfma_supported(L.oc, L.k, M) ? weak_grad_mfma_workspace(L.oc, L.k, M) : 0;
    if (need_dw > 0 && (!ws || ws_bytes < need_dw || !aligned16(ws))) return QEFT_ERR_WORKSPACE;
    // room for the partial tiles of a row split of dX: that split fills a sparse last round of tiles better than the
    // weak gradient's strips do, so it goes first (the strips' partial sums reuse the same bytes afterwards)
    // (a 3-bit layer: room for its fp16 copy - without it dX would take the slow general kernel - and, beyond that, for
    // the copy's own split; qeft_linear_bwd_dx uses what it is given)
    size_t need_dx = gemm_dx_supported(L, M) ? gemm_dx_split_workspace(L, M) : 0;
    if (dense_copy_applies(L, M)) need_dx = dense_copy_bytes(L);
    const bool split = need_dx > 0 && ws && aligned16(ws) && ws_bytes >= need_dx;
    if (!split && gemm_dx_dw_supported(L, M))
        return hip_status(gemm_dx_dw(L, (const __half*)dY, M, lddy, (__half*)dX, lddx, (const __half*)Xw, ldxw, dW,
                                     out_dtype == QEFT_DTYPE_F32, accumulate != 0, ws, (hipStream_t)stream));
    st = qeft_linear_bwd_dx(desc, w, dY, M, lddy, dX, lddx, split ? ws : nullptr, split ? ws_bytes : 0, stream);
    if (st != QEFT_OK) return st;
    return qeft_weak_grad(desc, dY, M, lddy, Xw, ldxw, dW, out_dtype, accumulate, ws, ws_bytes, stream);
}

const char* qeft_status_string(int status) {
    switch (status) {
        case QEFT_OK: return "ok";
        case QEFT_ERR_NULL: return "a required pointer is NULL";
        case QEFT_ERR_SHAPE: return "invalid shape or leading dimension";
        case QEFT_ERR_BITS: return "bits must be 3 or 4";
        case QEFT_ERR_ALIGN: return "pointer not 16-byte aligned or leading dimension not a multiple of 8";
        case QEFT_ERR_WORKSPACE: return "workspace missing or too small";
        case QEFT_ERR_UNSUPPORTED: return "unsupported layout, dtype or operation";
        case QEFT_ERR_HIP: return "HIP runtime error at launch";
        default: return "unknown status";
    }
}

}  // extern "C"
