/*
 * qeft.h - C ABI of the MI355X (gfx950) library for QEFT's fused mixed-precision
 * linear layer (arxiv 2410.08661).
 *
 * One linear layer with OC output and IC input channels is stored as three
 * components (paper Sec. 3.1): a dense low-bit code matrix over the Kq = IC - k
 * non-weak input channels, one fp16 (scale, zero-point) pair per group of g
 * adjacent non-weak channels of a row, and the k "weak" input channels kept in
 * fp16.  After the offline global reordering (Sec. 3.2) the weak channels are
 * contiguous; in this library they are the LAST k input channels, so that
 *
 *     W[o][j]      = scale[o][j/g] * (code[o][j] - zero[o][j/g])     j <  Kq
 *     W[o][Kq + c] = weak[o][c]                                      c <  k
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers owned by the caller; the library
 *     allocates nothing and never synchronises.  Its only state is a set of process-wide flags "the
 *     shared-memory limit of kernel X has been raised" (plain static booleans, set on a kernel's first
 *     launch and never cleared; two threads racing on one write the same value; they assume one GPU per
 *     process, the way this library is meant to be deployed).  Work is enqueued
 *     on `stream` (a hipStream_t passed as void*; NULL = the default stream) and
 *     ordered only by that stream.
 *   - Matrices are row-major with an explicit leading dimension in ELEMENTS.
 *     Activations and gradients are fp16; accumulation is fp32.
 *   - Return value: QEFT_OK or a negative qeft_status.  All argument checks run
 *     before anything is launched, so a failing call has no effect.  M == 0 is a
 *     valid no-op.  k == 0 (nothing weak) and k == IC (nothing quantized) are valid.
 */
#ifndef QEFT_H
#define QEFT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QEFT_OK = 0,
    QEFT_ERR_NULL = -1,        /* a required pointer is NULL                                   */
    QEFT_ERR_SHAPE = -2,       /* OC, IC, g <= 0 or above QEFT_MAX_DIM; k outside [0, IC]; M < 0 or above QEFT_MAX_DIM; ld < row width */
    QEFT_ERR_BITS = -3,        /* bits is not 3 or 4                                           */
    QEFT_ERR_ALIGN = -4,       /* pointer not 16-byte aligned, or ld not a multiple of 8       */
    QEFT_ERR_WORKSPACE = -5,   /* workspace missing or smaller than qeft_workspace_bytes()     */
    QEFT_ERR_UNSUPPORTED = -6, /* unknown layout / dtype / op, or a combination not implemented */
    QEFT_ERR_HIP = -7          /* the HIP runtime reported an error at launch                  */
} qeft_status;

/* Largest OC, IC, group size and number of rows M a call accepts (index arithmetic in the kernels is 32-bit per tile
 * and the host's tile and workspace counts are kept well inside 64 bits); larger values are QEFT_ERR_SHAPE, and
 * qeft_workspace_bytes / qeft_sensitivity_workspace report 0 for them.  (qeft_sensitivity takes up to 2^31 tokens.) */
#define QEFT_MAX_DIM (1 << 24)

/* How the codes of a row are laid out in its 32-bit words.
 *   QEFT_LAYOUT_CANONICAL  whole codes per word: 8 four-bit or 10 three-bit codes (bits 30..31 zero).
 *   QEFT_LAYOUT_DENSE3     3-bit only: the row is one bit string, code j at bits 3j .. 3j+2 of the row
 *                          (bit b of the row = bit b % 32 of word b / 32), 32 codes in 3 words, codes may
 *                          straddle words: 3.0 bits per quantized weight, the storage that the 3-bit model
 *                          sizes of the paper's Tab. 5 correspond to.  Every entry point takes either layout
 *                          (decode, M <= 16: a kernel of its own when the padded row holds whole groups, i.e.
 *                          12 * G <= row_stride_words, which every Kq that is a multiple of 128 satisfies;
 *                          larger M and the backward pass: as for all 3-bit layers, the tensor-core kernels on
 *                          an fp16 copy in the caller's workspace, see qeft_workspace_bytes, or the slow
 *                          general kernels without one). */
enum { QEFT_LAYOUT_CANONICAL = 0, QEFT_LAYOUT_DENSE3 = 1 };

/* Description of one layer (plain data, passed by pointer, host memory). */
typedef struct {
    int32_t out_features; /* OC                                                     */
    int32_t in_features;  /* IC, in reordered channel order (weak channels last)    */
    int32_t n_weak;       /* k, number of fp16 weak input channels, 0 <= k <= IC    */
    int32_t bits;         /* 4 or 3                                                 */
    int32_t group_size;   /* g, quantized columns sharing one (scale, zero) pair    */
    int32_t layout;       /* QEFT_LAYOUT_CANONICAL, or QEFT_LAYOUT_DENSE3 (bits == 3 only) */
} qeft_desc_t;

/* Sizes derived from a description (host memory). */
typedef struct {
    int64_t kq;               /* IC - k                                              */
    int64_t n_groups;         /* G = ceil(Kq / g)                                    */
    int64_t words_per_row;    /* ceil(Kq / 8) for 4-bit, ceil(Kq / 10) for 3-bit, ceil(3 Kq / 32) dense 3-bit */
    int64_t row_stride_words; /* words_per_row rounded up to a multiple of 16 (64 B) */
    int64_t group_stride;     /* G rounded up to a multiple of 8: row pitch of scales/zeros */
    size_t qweight_bytes;     /* OC * row_stride_words * 4                           */
    size_t scales_bytes;      /* OC * group_stride * 2                               */
    size_t zeros_bytes;       /* OC * group_stride * 2                               */
    size_t weak_bytes;        /* OC * k * 2                                          */
} qeft_layout_t;

/* The stored layer: four device pointers, borrowed for the duration of a call.
 *   qweight uint32 [OC][row_stride_words]  QEFT_LAYOUT_CANONICAL: code i of a word at bits
 *                                          [b*i, b*i+b), lowest column first; 8 codes per word
 *                                          for 4-bit, 10 for 3-bit (bits 30..31 zero).
 *                                          QEFT_LAYOUT_DENSE3: see above.  Row padding words
 *                                          (and bits past the last code) are zero.
 *   scales  fp16   [OC][group_stride]      entries past G are zero
 *   zeros   fp16   [OC][group_stride]      any fp16 value; qeft_pack writes integers
 *   weak    fp16   [OC][k]                 the trainable block; the caller's optimizer
 *                                          may update it between calls.
 * A pointer may be NULL only when its component is empty (Kq == 0 or k == 0). */
typedef struct {
    void* qweight;
    void* scales;
    void* zeros;
    void* weak;
} qeft_weight_t;

enum { QEFT_OP_FWD = 0, QEFT_OP_BWD_DX = 1, QEFT_OP_WEAK_GRAD = 2, QEFT_OP_FWD_IRREGULAR = 3, QEFT_OP_BWD_DX_IRREGULAR = 4,
       QEFT_OP_BWD = 5 };
enum { QEFT_DTYPE_F16 = 0, QEFT_DTYPE_F32 = 1 };

/* Component sizes of the stored form (Sec. 3.1).  Host only, pure. */
int qeft_layout(const qeft_desc_t* desc, qeft_layout_t* out);

/* Offline conversion of an fp16 weight into the stored form (Sec. 3.1; the data-free
 * quantizer is the paper's min-max round-to-nearest group quantization, Sec. 6.1 and
 * App. C).  W is fp16 [OC][ldw] on the device, columns already in reordered order.
 * Per row and group, in fp32: lo = min(0, min w), hi = max(0, max w),
 * s = fp16((hi - lo) / qmax) (1 if the group is all zero), z = clip(rint(-lo / s)),
 * code = clip(rint(w / s) + z), round-half-to-even.  The last k columns are copied to
 * out->weak.  Writes every byte of the four output buffers, padding included. */
int qeft_pack(const qeft_desc_t* desc, const void* W, int64_t ldw,
              const qeft_weight_t* out, void* stream);

/* The same conversion with the paper's group-wise grid search with truncation (Sec. 3.1): for every
 * (row, group), candidate i = 0 .. n_grid-1 shrinks the min-max range [lo, hi] to [p lo, p hi],
 * p = 1 - i * shrink_step, derives (s, z) from it by qeft_pack's rules, and the candidate with the
 * smallest squared weight error sum (w - s (q - z))^2 is kept (the first one on ties; candidate 0 is
 * qeft_pack's result, so no group gets worse).  The paper fixes neither the grid nor the arithmetic.
 * (s, z, codes) of a candidate are taken in fp32 with one rounding per operation, like qeft_pack's; the
 * error is summed in fp32 (eight consecutive columns at a time, then a tree over those sums), so between
 * candidates whose errors agree to about 1e-5 relative either may be kept.  n_grid >= 1,
 * (n_grid - 1) * shrink_step < 1.  This kernel needs group_size % 8 == 0, group_size <= 128 and
 * Kq % 8 == 0 (else QEFT_ERR_UNSUPPORTED).  The OPTQ step that follows in the paper needs calibration
 * data and is not part of this library: qeft_pack_codes takes its output. */
int qeft_pack_search(const qeft_desc_t* desc, const void* W, int64_t ldw, int n_grid, float shrink_step,
                     const qeft_weight_t* out, void* stream);

/* Build the stored form from already chosen codes (uint8 [OC][Kq], device) and
 * parameters (scales, zeros fp16 [OC][G] compact; weak fp16 [OC][k]): bit-packs the codes
 * and copies scales / zeros / weak into the padded stored arrays.  For quantizers
 * other than the built-in one (the paper's grid search + OPTQ, Sec. 3.1). */
int qeft_pack_codes(const qeft_desc_t* desc, const uint8_t* codes, const void* scales,
                    const void* zeros, const void* weak, const qeft_weight_t* out, void* stream);

/* Inverse of qeft_pack_codes: codes uint8 [OC][Kq], scales/zeros fp16 [OC][G], weak fp16
 * [OC][k], all device buffers of the caller.  Any output pointer may be NULL to skip it. */
int qeft_unpack(const qeft_desc_t* desc, const qeft_weight_t* w, uint8_t* codes,
                void* scales, void* zeros, void* weak, void* stream);

/* Bytes of device workspace an operation can use for M rows (0 if none).  QEFT_OP_WEAK_GRAD and the
 * irregular operations require theirs; those of QEFT_OP_FWD / QEFT_OP_BWD_DX are optional (NULL is always valid,
 * a workspace that is given must be 16-byte aligned and large enough, else QEFT_ERR_ALIGN / QEFT_ERR_WORKSPACE).
 * QEFT_OP_FWD / QEFT_OP_BWD_DX, 4-bit layers at M > 16 whose GEMM would leave compute units idle: split tiles *
 * splits * 128 KiB (one 256 x 256 fp16 partial tile per split).  With it the contraction range (input channels for
 * the forward, weight rows for the input gradient) of those tiles is split over several workgroups, partial tiles are
 * stored as fp16 and summed in fp32 by a second kernel (one extra fp16 rounding per split).  Two cases: fewer than
 * 160 output tiles - every tile, up to 16 splits (forward of 1024 x 8192 at M = 2048: 46 us against 150 us); or a
 * last round of tiles that fills at most half of the compute units - those tiles only, up to 8 splits, at most
 * 32 MiB (forward of 5120 x 13824 at M = 4096, 320 tiles on 256 units: 515 us against 651 us).
 * QEFT_OP_FWD / QEFT_OP_BWD_DX report OC * IC * 2 bytes for 3-bit layers
 * at M > 16 (plus the partial tiles of a split of the copy's columns or rows as above, used when the whole
 * amount is given): with that workspace (16-byte aligned) the call dequantizes the layer once into it as fp16 and
 * runs the tensor-core kernels on the copy - the paper's own training path, dequantize then a dense product
 * (Sec. 4.3, App. A.2) - and without it (ws NULL) the slow general kernel; a workspace that is too small is
 * QEFT_ERR_WORKSPACE.  The copy is rewritten by every call (the weak block may have changed).
 * QEFT_OP_BWD (qeft_linear_bwd): the larger of QEFT_OP_WEAK_GRAD's amount, which that call requires, and
 * QEFT_OP_BWD_DX's, which it uses when given (the two steps use the workspace one after the other). */
size_t qeft_workspace_bytes(const qeft_desc_t* desc, int op, int64_t M);

/* Forward of the fused layer (Sec. 3.2.1): Y = X[:, :Kq] . dq(Q)^T + X[:, Kq:] . weak^T in
 * one pass.  X fp16 [M][ldx] (ldx >= IC), Y fp16 [M][ldy] (ldy >= OC).  M <= 16 runs a
 * bandwidth-bound matrix-vector kernel, large M a tiled MFMA GEMM; for the token counts in between (up to
 * about 100, depending on the layer) several 16-token passes of the former where a host-side time model puts
 * them ahead of a GEMM that would fill only a fraction of the GPU.  ws / ws_bytes: optional, see
 * qeft_workspace_bytes (4-bit layers: partial tiles of a split launch; 3-bit layers: the fp16 copy and,
 * beyond it, the partial tiles of its split); NULL / 0 is always valid. */
int qeft_linear_fwd(const qeft_desc_t* desc, const qeft_weight_t* w, const void* X, int64_t M,
                    int64_t ldx, void* Y, int64_t ldy, void* ws, size_t ws_bytes, void* stream);

/* Forward of n (1 .. QEFT_MAX_GROUP) layers that read the same input, Y_i = X . W_i^T for each:
 * the query / key / value projections, or gate and up (Sec. 3.2.1; the weak columns are chosen
 * from the statistics of the layer's input, Sec. 3.1, so layers that share an input share
 * them).  The layers must agree in in_features, n_weak, bits, layout and group_size; out_features may
 * differ.  descs, w, Y and ldy are host arrays of n entries (w[i]'s device pointers and the
 * device buffer Y[i] fp16 [M][ldy[i]] are borrowed for the call).  Results equal those of n
 * qeft_linear_fwd calls up to summation order; decode-sized M runs them as one launch. */
#define QEFT_MAX_GROUP 4
int qeft_linear_fwd_group(int n, const qeft_desc_t* descs, const qeft_weight_t* w, const void* X,
                          int64_t M, int64_t ldx, void* const* Y, const int64_t* ldy, void* stream);

/* Input gradient through the full mixed weight (Sec. 3.3): dX = dY . W, i.e.
 * dX[:, :Kq] = dY . dq(Q) and dX[:, Kq:] = dY . weak (the weak block's current values).
 * dY fp16 [M][lddy] (lddy >= OC), dX fp16 [M][lddx] (lddx >= IC). */
int qeft_linear_bwd_dx(const qeft_desc_t* desc, const qeft_weight_t* w, const void* dY, int64_t M,
                       int64_t lddy, void* dX, int64_t lddx, void* ws, size_t ws_bytes, void* stream);

/* The layer whose weak columns stay at arbitrary input channels: the attention output
 * projection, which the offline reordering cannot reach, uses the mixed-precision format
 * without reordering and brings its activations into order on the fly (Sec. 3.2, last
 * paragraph; Limitations).  The stored form is the same as everywhere else - the non-weak
 * channels in ascending order, then the k weak ones - and perm (int32 [IC], device) names the
 * original input channel of every stored column.  X and dX are in ORIGINAL channel order:
 *     Y[m][o] = sum_j X[m][perm[j]] * W[o][j]        dX[m][perm[j]] = sum_o dY[m][o] * W[o][j]
 * perm must be a permutation of 0 .. IC-1 (entries are clamped to that range; a table that is
 * not a permutation gives unspecified values, never an access outside X / dX).  Both calls
 * need qeft_workspace_bytes(desc, QEFT_OP_FWD_IRREGULAR / QEFT_OP_BWD_DX_IRREGULAR, M) bytes of
 * device workspace, 16-byte aligned, for the gathered activations / the un-scattered gradient
 * (the forward of a 4-bit layer with M <= 4 gathers inside the matrix-vector kernel and does not touch it;
 * perm must be 16-byte aligned).
 * For the weak block's gradient, call qeft_weak_grad on the weak activations gathered by the
 * caller (X[:, perm[Kq:]], compact [M][k]). */
int qeft_linear_fwd_irregular(const qeft_desc_t* desc, const qeft_weight_t* w, const int32_t* perm,
                              const void* X, int64_t M, int64_t ldx, void* Y, int64_t ldy,
                              void* ws, size_t ws_bytes, void* stream);
int qeft_linear_bwd_dx_irregular(const qeft_desc_t* desc, const qeft_weight_t* w, const int32_t* perm,
                                 const void* dY, int64_t M, int64_t lddy, void* dX, int64_t lddx,
                                 void* ws, size_t ws_bytes, void* stream);

/* ---- one-time preparation: global weak columns and offline reordering (Sec. 3.2, App. B) ----
 *
 * qeft_sensitivity: the diagonal of the Hessian of a layer's input, out[j] = (2 / n_batch) *
 * sum_t X[t][j]^2 (fp32), for X fp16 [tokens][ldx] holding n_batch sequences one after the other;
 * d % 8 == 0.  Needs qeft_sensitivity_workspace(d, tokens) bytes of workspace.
 *
 * qeft_vote: the k entries of s (fp32 [d], device) with the largest values - equal values: lower
 * index first - are written to idx_out[0 .. k) in that order; if s_global is not NULL each of them
 * also adds s[j] / mean(s) to s_global[j] (a layer's vote, App. B).  With s_global == NULL this is a
 * plain top-k, which is also the final selection from the accumulated votes.
 *
 * qeft_weak_order: perm (int32 [d]) = the channels not in idx[0 .. k) in ascending order, then
 * idx[0 .. k) as given; idx must hold k distinct channels.
 *
 * qeft_reorder: out = A with its columns (axis 1) or rows (axis 0) taken in the order perm:
 * out[r][j] = A[r][perm[j]] or out[r][:] = A[perm[r]][:]; fp16 matrices [rows][ld], not in place.
 * Columns for the layers that read the hidden state, rows for the ones that write it (Fig. 3(b)).
 * Entries of perm are clamped to the valid range.  axis 0 needs cols % 8 == 0. */
size_t qeft_sensitivity_workspace(int32_t d, int64_t tokens);
int qeft_sensitivity(const void* X, int64_t tokens, int64_t ldx, int32_t d, int32_t n_batch, float* out,
                     void* ws, size_t ws_bytes, void* stream);
int qeft_vote(const float* s, int32_t d, int32_t k, int32_t* idx_out, float* s_global, void* stream);
int qeft_weak_order(const int32_t* idx, int32_t k, int32_t d, int32_t* perm, void* stream);
int qeft_reorder(const void* A, int64_t rows, int64_t cols, int64_t lda, const int32_t* perm, int axis,
                 void* out, int64_t ldo, void* stream);

/* QEFT merging (Sec. 5): the update of a fine-tuned weak block, tuned - base (both fp16 [OC][k],
 * compact), is added to another model's weight of the same layer: with idx (int32 [k], device) to
 * the columns idx[c] of a full-precision target fp16 [OC][ldt] with target_cols columns, with
 * idx == NULL to columns 0 .. k-1 of target (the target's own weak block: pass its pointer and
 * ldt = k).  fp32 arithmetic, one rounding to fp16 per element.  idx entries must be distinct
 * (they are clamped to the target's width). */
int qeft_merge_weak(const void* tuned, const void* base, int64_t out_features, int32_t k, const int32_t* idx,
                    void* target, int64_t ldt, int32_t target_cols, void* stream);

/* Weight gradient of the weak block only (Sec. 3.3, Eq. 5): dW[o][c] = sum_m dY[m][o] * Xw[m][c].
 * Xw fp16 [M][ldxw] holds the k weak activations of each token: either a view into X
 * (pointer X + Kq, ldxw = ldx) or the compact copy saved for backward (ldxw = k).
 * dW is [OC][k], fp16 or fp32 by out_dtype; accumulate != 0 adds to dW instead of
 * overwriting it (gradient accumulation, Tab. 4).  Needs a workspace. */
int qeft_weak_grad(const qeft_desc_t* desc, const void* dY, int64_t M, int64_t lddy,
                   const void* Xw, int64_t ldxw, void* dW, int out_dtype, int accumulate,
                   void* ws, size_t ws_bytes, void* stream);

/* The backward pass of one layer in one call (Sec. 3.3, Eq. 5): dX = dY . W through the full mixed weight and
 * dW (+)= dY^T . Xw for the weak block, arguments as in qeft_linear_bwd_dx and qeft_weak_grad.  The same kernels
 * run as in those two calls, and the results equal theirs bit for bit; what the call chooses is how they go out:
 *   - with room in ws for what qeft_linear_bwd_dx can use (qeft_workspace_bytes(desc, QEFT_OP_BWD, M), the larger
 *     of the two steps' amounts: the partial tiles of a row split of dX where that split applies, the fp16 copy of
 *     a 3-bit layer - without which its dX takes the slow general kernel): dX with that workspace, then the weak
 *     gradient, as qeft_linear_bwd_dx with its workspace followed by qeft_weak_grad (the workspace serves one after
 *     the other);
 *   - else, where both steps take the tensor-core path and the weak block is at most 128 wide: ONE launch - the
 *     weak gradient's workgroups follow the dX tiles in the grid and are dispatched as compute units fall free, so
 *     they run in what the last round of tiles leaves idle (dX of 4096 x 11008 at M = 4096: 688 tiles on 256 units;
 *     350 us against 363 us for the two calls); results as qeft_linear_bwd_dx without workspace followed by
 *     qeft_weak_grad;
 *   - else the two calls one after the other, dX without workspace.
 * ws / ws_bytes: at least qeft_workspace_bytes(desc, QEFT_OP_WEAK_GRAD, M) bytes, 16-byte aligned, required as for
 * qeft_weak_grad (QEFT_ERR_WORKSPACE before anything is launched); more than that is optional.
 * n_weak == 0: only dX is computed, without workspace (Xw, dW, ws may be NULL). */
int qeft_linear_bwd(const qeft_desc_t* desc, const qeft_weight_t* w, const void* dY, int64_t M, int64_t lddy,
                    void* dX, int64_t lddx, const void* Xw, int64_t ldxw, void* dW, int out_dtype, int accumulate,
                    void* ws, size_t ws_bytes, void* stream);

/* qeft_weak_grad for callers that cannot allocate and cannot hand over a workspace: code under HIP graph
 * capture, tight training or serving loops, harnesses that forbid hipMalloc.  Same arguments without ws, same
 * kernels and bit-identical results; the partial sums of the token split go to a device array inside the
 * library (QEFT_NOALLOC_SCRATCH_BYTES per GPU, held until the process ends) instead.  The call allocates
 * nothing and frees nothing.
 *   - QEFT_ERR_WORKSPACE when qeft_workspace_bytes(desc, QEFT_OP_WEAK_GRAD, M) exceeds
 *     QEFT_NOALLOC_SCRATCH_BYTES (all Llama-2 7B / 13B / 70B layer shapes fit); QEFT_ERR_UNSUPPORTED for the
 *     shapes qeft_weak_grad runs on its general kernel (M < 64, k > 256, k or OC not a multiple of 8) - it
 *     needs no workspace for those, call it instead.
 *   - Uses the array of the device that is current at the call, which must be the stream's device.
 *   - All calls on one GPU share that GPU's array: calls whose execution may overlap (different streams)
 *     race on it.  Calls ordered on one stream are safe; the buffer's previous contents are never read. */
#define QEFT_NOALLOC_SCRATCH_BYTES (14u * 1024u * 1024u)
int qeft_weak_grad_noalloc(const qeft_desc_t* desc, const void* dY, int64_t M, int64_t lddy,
                           const void* Xw, int64_t ldxw, void* dW, int out_dtype, int accumulate, void* stream);

/* Static, never NULL. */
const char* qeft_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* QEFT_H */
