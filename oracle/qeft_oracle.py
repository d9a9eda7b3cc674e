"""CPU oracle for QEFT's mixed-precision linear layer.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain definition that the HIP library is checked against.
Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may
import it; the product path never does, and it shares no code with the HIP path.

What it computes (paper sections in brackets):

* The stored form of one linear layer has three parts [Sec. 3.1]: a dense
  low-bit code matrix over the IC-k non-weak input channels, one (scale,
  zero-point) pair per group of g adjacent non-weak channels of a row, and the
  k weak input channels kept as an FP16 block.  After the offline global
  reordering the weak channels are contiguous [Sec. 3.2]; here they are the last
  k input channels.
* Forward [Sec. 3.2.1]: dequantize the codes, multiply with the activations,
  then add the product of the FP16 weak block with its activations:
      Y = X[:, :Kq] . dq(Q)^T + X[:, Kq:] . W_weak^T
* Backward [Sec. 3.3, Eq. 5]: dX = dY . W through the full mixed weight, and a
  weight gradient for the weak block only: dW_weak = dY^T . X[:, Kq:].
* Quantizer: the group-wise grid search with truncation of [Sec. 3.1] (quantize_search; the
  grid is this build's reading) and the paper's data-free fallback, min-max round-to-nearest per group
  [Sec. 6.1 (70B setting), App. C "Comparison of Quantization Methods",
  App. C "Quantization Cost"].

Arithmetic: everything that is a real number is float64 here (dequantized
weights s*(q-z) are exact in float64, sums carry ~1e-16 relative error).  The
one exception is the quantizer: its decisions (scale, zero-point, code) are
integers taken from floating point, so they are taken in IEEE float32, the
precision the kernel uses, with round-half-to-even.

Parity status: every function below is pinned by tests/test_oracle_*.py against
something other than itself (hand-written bit patterns, closed forms from the
paper's tables, exact-rational brute force, reductions to a library GEMM,
adjoint identities, known-answer quantization grids).
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "layout", "pack_codes", "unpack_codes", "pack_codes_dense3", "unpack_codes_dense3", "quantize_rtn", "codes_for_params", "search_candidates", "quantize_search", "dequantize",
    "stored_order", "linear_fwd_irregular", "linear_bwd_dx_irregular",
    "sensitivity", "top_k", "vote", "global_weak_columns", "reorder", "merge_weak",
    "linear_fwd", "linear_bwd_dx", "weak_grad", "round_fp16",
    "fwd_samples", "bwd_dx_samples", "weak_grad_samples",
]


# --------------------------------------------------------------------------- layout
def layout(out_features: int, in_features: int, n_weak: int, bits: int, group_size: int, dense: bool = False) -> dict:
    """Sizes of the three stored components [Sec. 3.1].

    dense=True (3-bit only) is the second stored layout: a row's codes as one bit string with
    no unused bits, 3.0 bits per weight, which is what the model sizes of [Tab. 5] imply for
    the 3-bit models (see pack_codes_dense3).

    Kq = IC - k columns are quantized.  Groups of g adjacent quantized columns
    tile [0, Kq); the last one may be partial.  Codes are bit-packed into 32-bit
    words, 8 four-bit or 10 three-bit codes per word (two top bits unused), and
    each row is padded with zero words to a multiple of 16 words (64 bytes: the
    paper does not describe row padding; one 128-column step of 4-bit codes is 64 bytes).
    Scales and zero-points are stored as [OC][group_stride] with group_stride = G rounded
    up to a multiple of 8 (16-byte rows), padding zero.
    """
    if bits not in (3, 4):
        raise ValueError("bits must be 3 or 4")
    oc, ic, k, g = int(out_features), int(in_features), int(n_weak), int(group_size)
    if oc <= 0 or ic <= 0 or g <= 0 or not (0 <= k <= ic):
        raise ValueError("bad shape")
    if dense and bits != 3:
        raise ValueError("the dense layout is defined for 3-bit codes only")
    per = 8 if bits == 4 else 10
    kq = ic - k
    n_groups = -(-kq // g)
    words = -(-(3 * kq) // 32) if dense else -(-kq // per)
    stride = -(-words // 16) * 16
    gstride = -(-n_groups // 8) * 8
    return {
        "kq": kq, "n_groups": n_groups, "codes_per_word": 32.0 / 3.0 if dense else per,
        "words_per_row": words, "row_stride_words": stride, "group_stride": gstride,
        "qweight_bytes": oc * stride * 4,
        "scales_bytes": oc * gstride * 2,
        "zeros_bytes": oc * gstride * 2,
        "weak_bytes": oc * k * 2,
    }


# --------------------------------------------------------------------------- bit packing
def pack_codes(codes: np.ndarray, bits: int, row_stride_words: int) -> np.ndarray:
    """codes uint8 [OC][Kq] -> uint32 [OC][row_stride_words].

    Code number i of a word sits at bit position bits*i (lowest code first);
    column j of a row is code j % per of word j // per.
    """
    per = 8 if bits == 4 else 10
    codes = np.asarray(codes, dtype=np.uint8)
    oc, kq = codes.shape
    if kq and int(codes.max()) >= (1 << bits):
        raise ValueError("code out of range")
    out = np.zeros((oc, row_stride_words), dtype=np.uint32)
    for j in range(kq):
        out[:, j // per] |= codes[:, j].astype(np.uint32) << np.uint32(bits * (j % per))
    return out


def unpack_codes(qweight: np.ndarray, kq: int, bits: int) -> np.ndarray:
    """Inverse of pack_codes: uint32 [OC][stride] -> uint8 [OC][Kq]."""
    per = 8 if bits == 4 else 10
    qweight = np.asarray(qweight, dtype=np.uint32)
    oc = qweight.shape[0]
    mask = np.uint32((1 << bits) - 1)
    out = np.zeros((oc, kq), dtype=np.uint8)
    j = np.arange(kq)
    word_of, shift_of = j // per, (bits * (j % per)).astype(np.uint32)
    for r0 in range(0, oc, 1024):          # row blocks only bound the temporary's size
        blk = qweight[r0:r0 + 1024]
        out[r0:r0 + 1024] = ((blk[:, word_of] >> shift_of[None, :]) & mask).astype(np.uint8)
    return out


def pack_codes_dense3(codes: np.ndarray, row_stride_words: int) -> np.ndarray:
    """Dense 3-bit layout: codes uint8 [OC][Kq] -> uint32 [OC][row_stride_words].

    A row is one little-endian bit string: code j occupies bits 3j, 3j+1, 3j+2 of the row
    (lowest bit of the code first), bit b of the row is bit b % 32 of word b // 32.  32 codes
    fill exactly 3 words; a code may straddle two words.  Bits past 3 Kq are zero.
    [Tab. 5: the 3-bit model sizes correspond to 3.0 bits per quantized weight.]
    """
    codes = np.asarray(codes, dtype=np.uint8)
    oc, kq = codes.shape
    if kq and int(codes.max()) >= 8:
        raise ValueError("code out of range")
    bits = np.zeros((oc, row_stride_words * 32), dtype=np.uint8)
    for b in range(3):
        bits[:, b:3 * kq:3] = (codes >> b) & 1
    by = np.packbits(bits, axis=1, bitorder="little")            # byte i = bits 8i .. 8i+7
    return np.ascontiguousarray(by).view("<u4").astype(np.uint32).reshape(oc, row_stride_words)


def unpack_codes_dense3(qweight: np.ndarray, kq: int) -> np.ndarray:
    """Inverse of pack_codes_dense3: uint32 [OC][stride] -> uint8 [OC][Kq]."""
    qweight = np.ascontiguousarray(np.asarray(qweight, dtype=np.uint32)).astype("<u4")
    oc = qweight.shape[0]
    out = np.zeros((oc, kq), dtype=np.uint8)
    for r0 in range(0, oc, 1024):          # row blocks only bound the temporary's size
        bits = np.unpackbits(qweight[r0:r0 + 1024].view(np.uint8), axis=1, bitorder="little")[:, :3 * kq]
        out[r0:r0 + 1024] = bits[:, 0::3] | (bits[:, 1::3] << 1) | (bits[:, 2::3] << 2)
    return out


# --------------------------------------------------------------------------- quantizer
def quantize_rtn(w: np.ndarray, n_weak: int, bits: int, group_size: int):
    """Min-max round-to-nearest group quantization of the non-weak columns.

    w: float16 [OC][IC].  Returns (codes uint8 [OC][Kq], scales f16 [OC][G],
    zeros f16 [OC][G], weak f16 [OC][k]).

    Per row and per group J of g adjacent quantized columns, all in float32:
        lo = min(0, min_J w)    hi = max(0, max_J w)        (range contains 0)
        s  = fp16((hi - lo) / qmax);   s = 1, z = 0 when hi == lo;
             the smallest positive fp16 if the rounding gave 0
        z  = clip(rint((0 - lo) / s), 0, qmax)              (an integer, never -0)
        q  = clip(rint(w / s) + z, 0, qmax)
    with rint = round-half-to-even and qmax = 2^bits - 1, so that the stored
    weight is s * (q - z).
    """
    w = np.asarray(w)
    assert w.dtype == np.float16 and w.ndim == 2
    oc, ic = w.shape
    k, g = int(n_weak), int(group_size)
    kq = ic - k
    n_groups = -(-kq // g)
    qmax = np.float32((1 << bits) - 1)
    wf = w[:, :kq].astype(np.float32)
    codes = np.zeros((oc, kq), dtype=np.uint8)
    scales = np.zeros((oc, n_groups), dtype=np.float16)
    zeros = np.zeros((oc, n_groups), dtype=np.float16)
    tiny = np.float16(2.0 ** -24)
    for gi in range(n_groups):
        blk = wf[:, gi * g:min((gi + 1) * g, kq)]
        lo = np.minimum(np.float32(0), blk.min(axis=1)).astype(np.float32)
        hi = np.maximum(np.float32(0), blk.max(axis=1)).astype(np.float32)
        s32 = ((hi - lo) / qmax).astype(np.float32)
        flat = s32 == 0
        s16 = s32.astype(np.float16)
        s16 = np.where((s16 == 0) & ~flat, tiny, s16)
        s16 = np.where(flat, np.float16(1.0), s16).astype(np.float16)
        s = s16.astype(np.float32)
        z = np.clip(np.rint(((np.float32(0) - lo) / s).astype(np.float32)), np.float32(0), qmax).astype(np.float32)
        z = np.where(flat, np.float32(0), z).astype(np.float32)
        q = np.rint((blk / s[:, None]).astype(np.float32)).astype(np.float32) + z[:, None]
        q = np.clip(q, np.float32(0), qmax)
        codes[:, gi * g:gi * g + blk.shape[1]] = q.astype(np.uint8)
        scales[:, gi] = s16
        zeros[:, gi] = z.astype(np.float16)
    weak = np.ascontiguousarray(w[:, kq:])
    return codes, scales, zeros, weak


def _group_params(lo, hi, qmax):
    """(scale fp16, zero-point f32, flat) from a range, with quantize_rtn's rules (float32)."""
    tiny = np.float16(2.0 ** -24)
    s32 = ((hi - lo) / qmax).astype(np.float32)
    flat = s32 == 0
    s16 = s32.astype(np.float16)
    s16 = np.where((s16 == 0) & ~flat, tiny, s16)
    s16 = np.where(flat, np.float16(1.0), s16).astype(np.float16)
    s = s16.astype(np.float32)
    z = np.clip(np.rint(((np.float32(0) - lo) / s).astype(np.float32)), np.float32(0), qmax).astype(np.float32)
    z = np.where(flat, np.float32(0), z).astype(np.float32)
    return s16, z


def codes_for_params(w: np.ndarray, n_weak: int, bits: int, group_size: int, scales: np.ndarray, zeros: np.ndarray) -> np.ndarray:
    """Round-to-nearest codes of the non-weak columns under GIVEN group parameters [Sec. 3.1]:
    q = clip(rint(w / s) + z, 0, qmax) in float32, round-half-to-even, as in quantize_rtn.
    scales, zeros: [OC][G].  -> uint8 [OC][Kq]."""
    w = np.asarray(w)
    assert w.dtype == np.float16 and w.ndim == 2
    oc, ic = w.shape
    g = int(group_size)
    kq = ic - int(n_weak)
    f32 = np.float32
    qmax = f32((1 << bits) - 1)
    codes = np.zeros((oc, kq), dtype=np.uint8)
    for gi in range(-(-kq // g)):
        blk = w[:, gi * g:min((gi + 1) * g, kq)].astype(np.float32)
        sf = np.asarray(scales)[:, gi].astype(np.float32)
        zf = np.asarray(zeros)[:, gi].astype(np.float32)
        q = np.rint((blk / sf[:, None]).astype(np.float32)).astype(np.float32) + zf[:, None]
        codes[:, gi * g:gi * g + blk.shape[1]] = np.clip(q, f32(0), qmax).astype(np.uint8)
    return codes


def search_candidates(w: np.ndarray, n_weak: int, bits: int, group_size: int, n_grid: int, shrink_step: float):
    """Every candidate of the group-wise grid search with truncation [Sec. 3.1], scored.

    The paper names a grid search per group that minimizes the squared weight error after the
    range is truncated; it gives neither the grid nor a precision.  Reading taken here: candidate
    i (i = 0 .. n_grid-1) shrinks the group's min-max range [lo, hi] (0 included, as in
    quantize_rtn) to [p_i lo, p_i hi] with p_i = 1 - i * shrink_step, derives (s, z) from that
    range by quantize_rtn's rules and quantizes with them.  Those are integer decisions taken
    from floating point, so they are IEEE float32 with one rounding per operation, as in
    quantize_rtn.  The score is a real number and is taken as such:
        E_i = sum_j (w_j - s (q_j - z))^2        in float64, a plain sum.
    Returns (scales f16 [n_grid][OC][G], zeros f32 [n_grid][OC][G], err f64 [n_grid][OC][G]).
    """
    w = np.asarray(w)
    assert w.dtype == np.float16 and w.ndim == 2
    oc, ic = w.shape
    k, g = int(n_weak), int(group_size)
    kq = ic - k
    f32 = np.float32
    assert n_grid >= 1 and f32(n_grid - 1) * f32(shrink_step) < f32(1)
    n_groups = -(-kq // g)
    qmax = f32((1 << bits) - 1)
    wf = w[:, :kq].astype(np.float32)
    s_all = np.zeros((n_grid, oc, n_groups), dtype=np.float16)
    z_all = np.zeros((n_grid, oc, n_groups), dtype=np.float32)
    e_all = np.zeros((n_grid, oc, n_groups), dtype=np.float64)
    for gi in range(n_groups):
        blk = wf[:, gi * g:min((gi + 1) * g, kq)]
        lo0 = np.minimum(f32(0), blk.min(axis=1)).astype(np.float32)
        hi0 = np.maximum(f32(0), blk.max(axis=1)).astype(np.float32)
        for i in range(n_grid):
            p = f32(f32(1) - f32(f32(i) * f32(shrink_step)))
            lo, hi = (p * lo0).astype(np.float32), (p * hi0).astype(np.float32)
            s16, z = _group_params(lo, hi, qmax)
            sf = s16.astype(np.float32)
            q = np.clip(np.rint((blk / sf[:, None]).astype(np.float32)).astype(np.float32) + z[:, None], f32(0), qmax)
            d = blk.astype(np.float64) - sf.astype(np.float64)[:, None] * (q.astype(np.float64) - z.astype(np.float64)[:, None])
            s_all[i, :, gi], z_all[i, :, gi], e_all[i, :, gi] = s16, z, np.sum(d * d, axis=1)
    return s_all, z_all, e_all


def quantize_search(w: np.ndarray, n_weak: int, bits: int, group_size: int, n_grid: int, shrink_step: float):
    """Group-wise grid search with truncation [Sec. 3.1]: per (row, group) the candidate of
    search_candidates with the smallest squared error; the first one on ties, so candidate 0
    (p = 1, plain min-max) is kept unless a truncated range is strictly better.  Any group size,
    any Kq.  Returns what quantize_rtn returns.

    Two candidates whose errors differ by less than rounding are both correct answers of the
    search; an implementation that sums in another precision or order may pick either, which is
    why a comparison against this function checks the error reached, not only the choice.
    """
    w = np.asarray(w)
    s_all, z_all, e_all = search_candidates(w, n_weak, bits, group_size, n_grid, shrink_step)
    oc, ic = w.shape
    k, g = int(n_weak), int(group_size)
    kq = ic - k
    n_groups = s_all.shape[2]
    f32 = np.float32
    qmax = f32((1 << bits) - 1)
    best = np.argmin(e_all, axis=0)                          # first minimum
    scales = np.take_along_axis(s_all, best[None], axis=0)[0]
    zf = np.take_along_axis(z_all, best[None], axis=0)[0]
    wf = w[:, :kq].astype(np.float32)
    codes = np.zeros((oc, kq), dtype=np.uint8)
    for gi in range(n_groups):
        blk = wf[:, gi * g:min((gi + 1) * g, kq)]
        sf = scales[:, gi].astype(np.float32)
        q = np.clip(np.rint((blk / sf[:, None]).astype(np.float32)).astype(np.float32) + zf[:, gi][:, None], f32(0), qmax)
        codes[:, gi * g:gi * g + blk.shape[1]] = q.astype(np.uint8)
    weak = np.ascontiguousarray(w[:, kq:])
    return codes, scales, zf.astype(np.float16), weak


# --------------------------------------------------------------------------- dequantize
def dequantize(codes: np.ndarray, scales: np.ndarray, zeros: np.ndarray,
               weak: np.ndarray, group_size: int) -> np.ndarray:
    """The full mixed weight W = [ s*(q - z) | W_weak ] as float64 [OC][IC]."""
    codes = np.asarray(codes, dtype=np.uint8)
    oc, kq = codes.shape
    k = weak.shape[1]
    w = np.empty((oc, kq + k), dtype=np.float64)
    s = np.asarray(scales).astype(np.float64)
    z = np.asarray(zeros).astype(np.float64)
    for j in range(kq):
        gi = j // group_size
        w[:, j] = s[:, gi] * (codes[:, j].astype(np.float64) - z[:, gi])
    w[:, kq:] = np.asarray(weak).astype(np.float64)
    return w


# --------------------------------------------------------------------------- the three products
def linear_fwd(w: np.ndarray, x: np.ndarray) -> np.ndarray:
    """Y = X . W^T  [Sec. 3.2.1].  w float64 [OC][IC], x [M][IC] -> float64 [M][OC]."""
    return np.asarray(x).astype(np.float64) @ w.T


def linear_bwd_dx(w: np.ndarray, dy: np.ndarray) -> np.ndarray:
    """dX = dY . W through the full mixed weight [Sec. 3.3].  dy [M][OC] -> [M][IC]."""
    return np.asarray(dy).astype(np.float64) @ w


def weak_grad(dy: np.ndarray, x_weak: np.ndarray) -> np.ndarray:
    """dW_weak = dY^T . X[:, weak]  [Sec. 3.3, Eq. 5].  -> float64 [OC][k]."""
    return np.asarray(dy).astype(np.float64).T @ np.asarray(x_weak).astype(np.float64)


# --------------------------------------------------------------------------- weak columns at arbitrary indices
# The attention output projection cannot be reordered offline [Sec. 3.2, last paragraph;
# Limitations]: its weak columns stay where the sensitivity analysis found them, and the
# mixed-precision format is used "without reordering": the stored layer holds the non-weak
# columns in ascending order (quantized, grouped over that compacted order) followed by the
# weak block, and the activations are brought into that order on the fly.
def stored_order(in_features: int, weak_idx) -> np.ndarray:
    """perm[j] = original input channel held at stored position j: the non-weak channels in
    ascending order, then the weak channels in the order given.  weak_idx: k distinct indices."""
    weak_idx = np.asarray(weak_idx, dtype=np.int64)
    assert weak_idx.ndim == 1 and len(set(weak_idx.tolist())) == len(weak_idx)
    assert len(weak_idx) == 0 or (weak_idx.min() >= 0 and weak_idx.max() < in_features)
    is_weak = np.zeros(in_features, dtype=bool)
    is_weak[weak_idx] = True
    return np.concatenate([np.nonzero(~is_weak)[0], weak_idx]).astype(np.int32)


def linear_fwd_irregular(w_stored: np.ndarray, perm: np.ndarray, x: np.ndarray) -> np.ndarray:
    """Forward with the weak columns at arbitrary indices: w_stored float64 [OC][IC] is the
    dequantized stored layer (columns in stored order), x [M][IC] is in ORIGINAL channel
    order.  Y[m][o] = sum_j x[m][perm[j]] * w_stored[o][j]."""
    x = np.asarray(x).astype(np.float64)
    return x[:, np.asarray(perm, dtype=np.int64)] @ w_stored.T


def linear_bwd_dx_irregular(w_stored: np.ndarray, perm: np.ndarray, dy: np.ndarray) -> np.ndarray:
    """dX in ORIGINAL channel order: dX[m][perm[j]] = sum_o dy[m][o] * w_stored[o][j]."""
    d = np.asarray(dy).astype(np.float64) @ w_stored
    out = np.empty_like(d)
    out[:, np.asarray(perm, dtype=np.int64)] = d
    return out


# --------------------------------------------------------------------------- global weak columns and reordering
# Which input channels are weak is decided once for the whole network [Sec. 3.2, App. B]: every
# layer ranks its input channels by the diagonal of the Hessian of its input, its k best vote
# with their sensitivity relative to the layer's mean, and the k channels with the largest
# accumulated vote win.  The model is then reordered offline so that they are contiguous.
def sensitivity(x: np.ndarray, n_batch: int) -> np.ndarray:
    """Diagonal of H = mean over the batch of 2 X_b^T X_b  [App. B; lambda_j of Sec. 3.1]:
    x [tokens][d] holds the n_batch sequences one after the other; -> float64 [d],
    s_j = (2 / n_batch) * sum_t x[t][j]^2."""
    x = np.asarray(x).astype(np.float64)
    return 2.0 * np.sum(x * x, axis=0) / float(n_batch)


def top_k(v: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest entries, largest first; equal values: lower index first."""
    v = np.asarray(v, dtype=np.float64)
    order = sorted(range(len(v)), key=lambda i: (-v[i], i))
    return np.array(order[:k], dtype=np.int32)


def vote(s_local: np.ndarray, k: int, s_global: np.ndarray) -> np.ndarray:
    """One layer's contribution [App. B]: its k most sensitive channels add their sensitivity
    divided by the layer's mean sensitivity to s_global (in place); returns those channels."""
    s_local = np.asarray(s_local, dtype=np.float64)
    chosen = top_k(s_local, k)
    layer_mean = float(np.mean(s_local))
    for j in chosen.tolist():
        s_global[j] += s_local[j] / layer_mean
    return chosen


def global_weak_columns(layer_inputs, k: int) -> np.ndarray:
    """layer_inputs: iterable of (x [tokens][d], n_batch), one per linear layer that reads the
    hidden state.  -> the k global weak channels, largest accumulated vote first."""
    s_global = None
    for x, n_batch in layer_inputs:
        s_local = sensitivity(x, n_batch)
        if s_global is None:
            s_global = np.zeros(len(s_local), dtype=np.float64)
        vote(s_local, k, s_global)
    return top_k(s_global, k)


def reorder(a: np.ndarray, perm: np.ndarray, axis: int) -> np.ndarray:
    """Offline reordering of one weight (or activation) matrix along `axis`: position j of the
    result holds index perm[j] of the original (columns for the layers that read the hidden state,
    rows for the ones that write it) [Sec. 3.2, Fig. 3(b)]."""
    return np.take(np.asarray(a), np.asarray(perm, dtype=np.int64), axis=axis)


def merge_weak(target: np.ndarray, tuned: np.ndarray, base: np.ndarray, idx=None) -> np.ndarray:
    """QEFT merging [Sec. 5, "QEFT merging"]: the update of the fine-tuned weak columns,
    Delta = A' - A, is added to the corresponding columns of another model's weight: to the
    columns idx of a full-precision target, or (idx None) to the target's own weak block.
    All fp16; the arithmetic is float32 with one rounding per operation, then one to fp16
    (a difference of two fp16 numbers is exact in float32)."""
    t = np.array(target, dtype=np.float16, copy=True)
    delta = np.asarray(tuned, dtype=np.float16).astype(np.float32) - np.asarray(base, dtype=np.float16).astype(np.float32)
    cols = np.arange(delta.shape[1]) if idx is None else np.asarray(idx, dtype=np.int64)
    t[:, cols] = (t[:, cols].astype(np.float32) + delta).astype(np.float32).astype(np.float16)
    return t


def round_fp16(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even to float16 (the dtype of Y, dX and optionally dW)."""
    return np.asarray(a, dtype=np.float64).astype(np.float16)


# --------------------------------------------------------------------------- sampled outputs
# At full benchmark sizes the whole product is too slow for a test; these compute
# single outputs one by one from the packed arrays: unpack the row (or column),
# dequantize it, take the dot product.
def _row(qweight, scales, zeros, weak, o, kq, bits, group_size):
    # bits == "3d" names the dense 3-bit layout
    codes = unpack_codes_dense3(qweight[o:o + 1], kq) if bits == "3d" else unpack_codes(qweight[o:o + 1], kq, bits)
    return dequantize(codes, scales[o:o + 1], zeros[o:o + 1], weak[o:o + 1], group_size)[0]


def fwd_samples(qweight, scales, zeros, weak, kq, bits, group_size, x, pairs):
    """Y[m, o] for each (m, o) in pairs."""
    out = np.empty(len(pairs), dtype=np.float64)
    rows = {}
    for i, (m, o) in enumerate(pairs):
        if o not in rows:
            rows[o] = _row(qweight, scales, zeros, weak, o, kq, bits, group_size)
        out[i] = np.dot(np.asarray(x[m]).astype(np.float64), rows[o])
    return out


def bwd_dx_samples(qweight, scales, zeros, weak, kq, bits, group_size, dy, pairs):
    """dX[m, c] for each (m, c) in pairs."""
    dense = bits == "3d"
    if not dense:
        per = 8 if bits == 4 else 10
        mask = (1 << bits) - 1
    out = np.empty(len(pairs), dtype=np.float64)
    cols = {}
    for i, (m, c) in enumerate(pairs):
        if c not in cols:
            if c < kq:
                if dense:   # the three bits 3c .. 3c+2 of the row's bit string
                    w0, sh = (3 * c) // 32, (3 * c) % 32
                    two = np.asarray(qweight[:, w0]).astype(np.uint64)
                    if sh > 29:
                        two = two | (np.asarray(qweight[:, w0 + 1]).astype(np.uint64) << np.uint64(32))
                    q = (two >> np.uint64(sh)) & np.uint64(7)
                else:
                    q = (np.asarray(qweight[:, c // per]).astype(np.uint32) >> np.uint32(bits * (c % per))) & np.uint32(mask)
                gi = c // group_size
                cols[c] = np.asarray(scales[:, gi]).astype(np.float64) * (
                    q.astype(np.float64) - np.asarray(zeros[:, gi]).astype(np.float64))
            else:
                cols[c] = np.asarray(weak[:, c - kq]).astype(np.float64)
        out[i] = np.dot(np.asarray(dy[m]).astype(np.float64), cols[c])
    return out


def weak_grad_samples(dy, x_weak, pairs):
    """dW_weak[o, c] for each (o, c) in pairs."""
    out = np.empty(len(pairs), dtype=np.float64)
    for i, (o, c) in enumerate(pairs):
        out[i] = np.dot(np.asarray(dy[:, o]).astype(np.float64), np.asarray(x_weak[:, c]).astype(np.float64))
    return out
