"""ctypes binding of libqeft.so: the same entry points as include/qeft.h.

Argument marshalling only.  `raw` exposes the C functions as they are (integers for
pointers), the functions below take torch tensors and pass `data_ptr()` and the current
HIP stream.  PyTorch is used for device memory and streams, nothing else; there is no
fallback path: if the library is missing the import fails.
"""
from __future__ import annotations

import ctypes as C
import os

import torch  # imported first on purpose: the library must bind to the HIP runtime torch loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqeft.so")

QEFT_OK = 0
QEFT_ERR_NULL, QEFT_ERR_SHAPE, QEFT_ERR_BITS, QEFT_ERR_ALIGN = -1, -2, -3, -4
QEFT_ERR_WORKSPACE, QEFT_ERR_UNSUPPORTED, QEFT_ERR_HIP = -5, -6, -7
QEFT_OP_FWD, QEFT_OP_BWD_DX, QEFT_OP_WEAK_GRAD, QEFT_OP_FWD_IRREGULAR, QEFT_OP_BWD_DX_IRREGULAR, QEFT_OP_BWD = 0, 1, 2, 3, 4, 5
QEFT_DTYPE_F16, QEFT_DTYPE_F32 = 0, 1
QEFT_LAYOUT_CANONICAL, QEFT_LAYOUT_DENSE3 = 0, 1


class qeft_desc_t(C.Structure):
    _fields_ = [("out_features", C.c_int32), ("in_features", C.c_int32), ("n_weak", C.c_int32),
                ("bits", C.c_int32), ("group_size", C.c_int32), ("layout", C.c_int32)]


class qeft_layout_t(C.Structure):
    _fields_ = [("kq", C.c_int64), ("n_groups", C.c_int64), ("words_per_row", C.c_int64),
                ("row_stride_words", C.c_int64), ("group_stride", C.c_int64), ("qweight_bytes", C.c_size_t),
                ("scales_bytes", C.c_size_t),
                ("zeros_bytes", C.c_size_t), ("weak_bytes", C.c_size_t)]


class qeft_weight_t(C.Structure):
    _fields_ = [("qweight", C.c_void_p), ("scales", C.c_void_p), ("zeros", C.c_void_p), ("weak", C.c_void_p)]


EXPORTS = {
    "qeft_layout": (C.c_int, [C.POINTER(qeft_desc_t), C.POINTER(qeft_layout_t)]),
    "qeft_pack": (C.c_int, [C.POINTER(qeft_desc_t), C.c_void_p, C.c_int64, C.POINTER(qeft_weight_t), C.c_void_p]),
    "qeft_pack_search": (C.c_int, [C.POINTER(qeft_desc_t), C.c_void_p, C.c_int64, C.c_int, C.c_float,
                                   C.POINTER(qeft_weight_t), C.c_void_p]),
    "qeft_pack_codes": (C.c_int, [C.POINTER(qeft_desc_t), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                  C.POINTER(qeft_weight_t), C.c_void_p]),
    "qeft_unpack": (C.c_int, [C.POINTER(qeft_desc_t), C.POINTER(qeft_weight_t), C.c_void_p, C.c_void_p, C.c_void_p,
                              C.c_void_p, C.c_void_p]),
    "qeft_workspace_bytes": (C.c_size_t, [C.POINTER(qeft_desc_t), C.c_int, C.c_int64]),
    "qeft_linear_fwd": (C.c_int, [C.POINTER(qeft_desc_t), C.POINTER(qeft_weight_t), C.c_void_p, C.c_int64, C.c_int64,
                                  C.c_void_p, C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p]),
    "qeft_linear_fwd_group": (C.c_int, [C.c_int, C.POINTER(qeft_desc_t), C.POINTER(qeft_weight_t), C.c_void_p, C.c_int64,
                                        C.c_int64, C.POINTER(C.c_void_p), C.POINTER(C.c_int64), C.c_void_p]),
    "qeft_linear_bwd_dx": (C.c_int, [C.POINTER(qeft_desc_t), C.POINTER(qeft_weight_t), C.c_void_p, C.c_int64,
                                     C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p]),
    "qeft_linear_fwd_irregular": (C.c_int, [C.POINTER(qeft_desc_t), C.POINTER(qeft_weight_t), C.c_void_p, C.c_void_p,
                                            C.c_int64, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p]),
    "qeft_linear_bwd_dx_irregular": (C.c_int, [C.POINTER(qeft_desc_t), C.POINTER(qeft_weight_t), C.c_void_p, C.c_void_p,
                                               C.c_int64, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p]),
    "qeft_sensitivity_workspace": (C.c_size_t, [C.c_int32, C.c_int64]),
    "qeft_sensitivity": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                   C.c_size_t, C.c_void_p]),
    "qeft_vote": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "qeft_weak_order": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "qeft_reorder": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_int, C.c_void_p, C.c_int64,
                               C.c_void_p]),
    "qeft_merge_weak": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
                                  C.c_void_p]),
    "qeft_weak_grad": (C.c_int, [C.POINTER(qeft_desc_t), C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int64,
                                 C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]),
    "qeft_linear_bwd": (C.c_int, [C.POINTER(qeft_desc_t), C.POINTER(qeft_weight_t), C.c_void_p, C.c_int64, C.c_int64, C.c_void_p,
                                  C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]),
    "qeft_weak_grad_noalloc": (C.c_int, [C.POINTER(qeft_desc_t), C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int64,
                                         C.c_void_p, C.c_int, C.c_int, C.c_void_p]),
    "qeft_status_string": (C.c_char_p, [C.c_int]),
}


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2410_08661_amd.build`")
    lib = C.CDLL(LIB_PATH)
    for name, (res, args) in EXPORTS.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


raw = _load()


class QeftError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {raw.qeft_status_string(status).decode()} ({status})")


def _check(status: int, where: str) -> None:
    if status != QEFT_OK:
        raise QeftError(status, where)


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def make_desc(out_features, in_features, n_weak, bits=4, group_size=128, layout=0) -> qeft_desc_t:
    return qeft_desc_t(out_features, in_features, n_weak, bits, group_size, layout)


def qeft_layout(desc: qeft_desc_t) -> qeft_layout_t:
    out = qeft_layout_t()
    _check(raw.qeft_layout(C.byref(desc), C.byref(out)), "qeft_layout")
    return out


class Weight:
    """The four device buffers of one stored layer (torch tensors own the memory)."""

    def __init__(self, desc: qeft_desc_t, device="cuda"):
        lay = qeft_layout(desc)
        self.desc, self.lay = desc, lay
        oc = desc.out_features
        self.qweight = torch.zeros((oc, lay.row_stride_words), dtype=torch.int32, device=device)
        self.scales = torch.zeros((oc, lay.group_stride), dtype=torch.float16, device=device)
        self.zeros = torch.zeros((oc, lay.group_stride), dtype=torch.float16, device=device)
        self.weak = torch.zeros((oc, desc.n_weak), dtype=torch.float16, device=device)

    def c_struct(self) -> qeft_weight_t:
        lay, d = self.lay, self.desc
        return qeft_weight_t(self.qweight.data_ptr() if lay.kq else None, self.scales.data_ptr() if lay.kq else None,
                             self.zeros.data_ptr() if lay.kq else None, self.weak.data_ptr() if d.n_weak else None)

    def nbytes(self) -> int:
        lay = self.lay
        return lay.qweight_bytes + lay.scales_bytes + lay.zeros_bytes + lay.weak_bytes


def qeft_pack(desc: qeft_desc_t, W: torch.Tensor, out: Weight | None = None) -> Weight:
    out = out or Weight(desc, W.device)
    ws = out.c_struct()
    _check(raw.qeft_pack(C.byref(desc), _ptr(W), W.stride(0), C.byref(ws), _stream()), "qeft_pack")
    return out


def qeft_pack_search(desc: qeft_desc_t, W: torch.Tensor, n_grid: int = 80, shrink_step: float = 0.01,
                     out: Weight | None = None) -> Weight:
    """qeft_pack with the group-wise grid search over truncated ranges."""
    out = out or Weight(desc, W.device)
    ws = out.c_struct()
    _check(raw.qeft_pack_search(C.byref(desc), _ptr(W), W.stride(0), int(n_grid), float(shrink_step), C.byref(ws),
                                _stream()), "qeft_pack_search")
    return out


def qeft_pack_codes(desc, codes, scales, zeros, weak, out: Weight | None = None) -> Weight:
    out = out or Weight(desc, weak.device if weak is not None else codes.device)
    ws = out.c_struct()
    _check(raw.qeft_pack_codes(C.byref(desc), _ptr(codes), _ptr(scales), _ptr(zeros), _ptr(weak), C.byref(ws),
                               _stream()), "qeft_pack_codes")
    return out


def qeft_unpack(desc, w: Weight):
    lay = w.lay
    dev = w.qweight.device
    codes = torch.empty((desc.out_features, lay.kq), dtype=torch.uint8, device=dev)
    scales = torch.empty((desc.out_features, lay.n_groups), dtype=torch.float16, device=dev)
    zeros, weak = torch.empty_like(scales), torch.empty_like(w.weak)
    ws = w.c_struct()
    _check(raw.qeft_unpack(C.byref(desc), C.byref(ws), _ptr(codes) if lay.kq else None,
                           _ptr(scales) if lay.kq else None, _ptr(zeros) if lay.kq else None,
                           _ptr(weak) if desc.n_weak else None, _stream()), "qeft_unpack")
    return codes, scales, zeros, weak


def _empty_rows(m: int, cols: int, dtype, device) -> torch.Tensor:
    """[m][cols] tensor whose leading dimension is padded to a multiple of 8 elements."""
    ld = (max(cols, 1) + 7) // 8 * 8
    return torch.empty((m, ld), dtype=dtype, device=device)[:, :cols]


def qeft_workspace_bytes(desc, op: int, M: int) -> int:
    return int(raw.qeft_workspace_bytes(C.byref(desc), op, M))


def _workspace(desc, op, M, device):
    n = qeft_workspace_bytes(desc, op, M)
    return (torch.empty(n, dtype=torch.uint8, device=device), n) if n else (None, 0)


def qeft_linear_fwd(desc, w: Weight, X: torch.Tensor, Y: torch.Tensor | None = None, ws=None) -> torch.Tensor:
    """ws: a uint8 device tensor of qeft_workspace_bytes(desc, QEFT_OP_FWD, M) bytes; None allocates one when the
    operation can use it (3-bit layers at M > 16), False passes none (the library then runs its general kernel)."""
    M = X.shape[0]
    if Y is None:
        Y = _empty_rows(M, desc.out_features, torch.float16, X.device)
    if ws is None:
        ws, _ = _workspace(desc, QEFT_OP_FWD, M, X.device)
    elif ws is False:
        ws = None
    wst = w.c_struct()
    _check(raw.qeft_linear_fwd(C.byref(desc), C.byref(wst), _ptr(X), M, X.stride(0) if M else desc.in_features,
                               _ptr(Y), Y.stride(0) if M else desc.out_features, _ptr(ws),
                               ws.numel() if ws is not None else 0, _stream()), "qeft_linear_fwd")
    return Y


class Group:
    """The host-side argument arrays of qeft_linear_fwd_group for a fixed set of layers and outputs
    (built once; a decode loop then only passes X)."""

    def __init__(self, descs, ws, Ys):
        n = len(descs)
        assert n == len(ws) == len(Ys) and n >= 1
        self.n = n
        self.descs = (qeft_desc_t * n)(*descs)
        self.wst = (qeft_weight_t * n)(*[w.c_struct() for w in ws])
        self.ys = (C.c_void_p * n)(*[_ptr(y) for y in Ys])
        self.ldy = (C.c_int64 * n)(*[y.stride(0) for y in Ys])
        self.keep = (list(ws), list(Ys))   # the device buffers the arrays point into
        self.Ys = list(Ys)


def qeft_linear_fwd_group(descs, ws, X: torch.Tensor, Ys=None, group: Group | None = None):
    """Forward of several layers that share the input X; returns the list of outputs."""
    M = X.shape[0]
    if group is None:
        if Ys is None:
            Ys = [_empty_rows(M, d.out_features, torch.float16, X.device) for d in descs]
        group = Group(descs, ws, Ys)
    _check(raw.qeft_linear_fwd_group(group.n, group.descs, group.wst, _ptr(X), M,
                                     X.stride(0) if M else group.descs[0].in_features, group.ys, group.ldy, _stream()),
           "qeft_linear_fwd_group")
    return group.Ys


def qeft_linear_bwd_dx(desc, w: Weight, dY: torch.Tensor, dX: torch.Tensor | None = None, ws=None) -> torch.Tensor:
    M = dY.shape[0]
    if dX is None:
        dX = _empty_rows(M, desc.in_features, torch.float16, dY.device)
    if ws is None:
        ws, _ = _workspace(desc, QEFT_OP_BWD_DX, M, dY.device)
    elif ws is False:
        ws = None
    wst = w.c_struct()
    _check(raw.qeft_linear_bwd_dx(C.byref(desc), C.byref(wst), _ptr(dY), M, dY.stride(0) if M else desc.out_features,
                                  _ptr(dX), dX.stride(0) if M else desc.in_features, _ptr(ws),
                                  ws.numel() if ws is not None else 0, _stream()), "qeft_linear_bwd_dx")
    return dX


def qeft_linear_fwd_irregular(desc, w: Weight, perm: torch.Tensor, X: torch.Tensor, Y: torch.Tensor | None = None,
                              ws=None) -> torch.Tensor:
    """Forward of a layer whose weak columns stay at arbitrary channels; perm int32 [IC] on the device."""
    M = X.shape[0]
    if Y is None:
        Y = _empty_rows(M, desc.out_features, torch.float16, X.device)
    if ws is None:
        ws, _ = _workspace(desc, QEFT_OP_FWD_IRREGULAR, M, X.device)
    wst = w.c_struct()
    _check(raw.qeft_linear_fwd_irregular(C.byref(desc), C.byref(wst), _ptr(perm), _ptr(X), M,
                                         X.stride(0) if M else desc.in_features, _ptr(Y),
                                         Y.stride(0) if M else desc.out_features, _ptr(ws),
                                         ws.numel() if ws is not None else 0, _stream()), "qeft_linear_fwd_irregular")
    return Y


def qeft_linear_bwd_dx_irregular(desc, w: Weight, perm: torch.Tensor, dY: torch.Tensor, dX: torch.Tensor | None = None,
                                 ws=None) -> torch.Tensor:
    M = dY.shape[0]
    if dX is None:
        dX = _empty_rows(M, desc.in_features, torch.float16, dY.device)
    if ws is None:
        ws, _ = _workspace(desc, QEFT_OP_BWD_DX_IRREGULAR, M, dY.device)
    wst = w.c_struct()
    _check(raw.qeft_linear_bwd_dx_irregular(C.byref(desc), C.byref(wst), _ptr(perm), _ptr(dY), M,
                                            dY.stride(0) if M else desc.out_features, _ptr(dX),
                                            dX.stride(0) if M else desc.in_features, _ptr(ws),
                                            ws.numel() if ws is not None else 0, _stream()),
           "qeft_linear_bwd_dx_irregular")
    return dX


def qeft_sensitivity(X: torch.Tensor, n_batch: int) -> torch.Tensor:
    """Diagonal of the layer input's Hessian, fp32 [d]."""
    tokens, d = X.shape
    out = torch.empty(d, dtype=torch.float32, device=X.device)
    n = int(raw.qeft_sensitivity_workspace(d, tokens))
    ws = torch.empty(max(n, 16), dtype=torch.uint8, device=X.device)
    _check(raw.qeft_sensitivity(_ptr(X), tokens, X.stride(0), d, int(n_batch), _ptr(out), _ptr(ws), ws.numel(), _stream()),
           "qeft_sensitivity")
    return out


def qeft_vote(s: torch.Tensor, k: int, s_global: torch.Tensor | None = None) -> torch.Tensor:
    """Top-k channels of s (int32 [k], largest first); with s_global their votes are added to it."""
    idx = torch.empty(k, dtype=torch.int32, device=s.device)
    _check(raw.qeft_vote(_ptr(s), s.numel(), int(k), _ptr(idx), _ptr(s_global), _stream()), "qeft_vote")
    return idx


def qeft_weak_order(idx: torch.Tensor, d: int) -> torch.Tensor:
    perm = torch.empty(d, dtype=torch.int32, device=idx.device)
    _check(raw.qeft_weak_order(_ptr(idx), idx.numel(), int(d), _ptr(perm), _stream()), "qeft_weak_order")
    return perm


def qeft_reorder(A: torch.Tensor, perm: torch.Tensor, axis: int) -> torch.Tensor:
    rows, cols = A.shape
    out = _empty_rows(rows, cols, torch.float16, A.device)
    _check(raw.qeft_reorder(_ptr(A), rows, cols, A.stride(0), _ptr(perm), int(axis), _ptr(out), out.stride(0), _stream()),
           "qeft_reorder")
    return out


def qeft_merge_weak(tuned: torch.Tensor, base: torch.Tensor, target: torch.Tensor, idx: torch.Tensor | None = None) -> torch.Tensor:
    """target[:, idx] (or target[:, :k]) += tuned - base, in place."""
    oc, k = tuned.shape
    _check(raw.qeft_merge_weak(_ptr(tuned), _ptr(base), oc, k, _ptr(idx), _ptr(target), target.stride(0), target.shape[1],
                               _stream()), "qeft_merge_weak")
    return target


def qeft_weak_grad(desc, dY: torch.Tensor, Xw: torch.Tensor, dW: torch.Tensor | None = None, accumulate=False,
                   out_dtype=torch.float32, ws=None) -> torch.Tensor:
    M = dY.shape[0]
    if dW is None:
        dW = torch.zeros((desc.out_features, desc.n_weak), dtype=out_dtype, device=dY.device)
    code = {torch.float16: QEFT_DTYPE_F16, torch.float32: QEFT_DTYPE_F32}[dW.dtype]
    if ws is None:
        ws, _ = _workspace(desc, QEFT_OP_WEAK_GRAD, M, dY.device)
    _check(raw.qeft_weak_grad(C.byref(desc), _ptr(dY), M, dY.stride(0) if M else desc.out_features, _ptr(Xw),
                              Xw.stride(0) if M else max(desc.n_weak, 8), _ptr(dW), code, int(bool(accumulate)),
                              _ptr(ws), ws.numel() if ws is not None else 0, _stream()), "qeft_weak_grad")
    return dW


def qeft_weak_grad_noalloc(desc, dY: torch.Tensor, Xw: torch.Tensor, dW: torch.Tensor, accumulate=False) -> torch.Tensor:
    """qeft_weak_grad without a workspace argument: the library's own per-GPU scratch array takes the partial sums.
    dW must be given (this call allocates nothing, here or in the library)."""
    M = dY.shape[0]
    code = {torch.float16: QEFT_DTYPE_F16, torch.float32: QEFT_DTYPE_F32}[dW.dtype]
    _check(raw.qeft_weak_grad_noalloc(C.byref(desc), _ptr(dY), M, dY.stride(0) if M else desc.out_features, _ptr(Xw),
                                      Xw.stride(0) if M else max(desc.n_weak, 8), _ptr(dW), code, int(bool(accumulate)),
                                      _stream()), "qeft_weak_grad_noalloc")
    return dW


def qeft_linear_bwd(desc, w: Weight, dY: torch.Tensor, Xw: torch.Tensor, dX: torch.Tensor | None = None,
                    dW: torch.Tensor | None = None, accumulate=False, out_dtype=torch.float32, ws=None):
    """dX and dW_weak of one layer in one call; returns (dX, dW).  ws: None allocates the weak gradient's workspace;
    a tensor of qeft_workspace_bytes(desc, QEFT_OP_BWD, M) bytes also lets dX split its rows where that pays."""
    M = dY.shape[0]
    if dX is None:
        dX = _empty_rows(M, desc.in_features, torch.float16, dY.device)
    if dW is None:
        dW = torch.zeros((desc.out_features, desc.n_weak), dtype=out_dtype, device=dY.device)
    code = {torch.float16: QEFT_DTYPE_F16, torch.float32: QEFT_DTYPE_F32}[dW.dtype]
    if ws is None:
        ws, _ = _workspace(desc, QEFT_OP_WEAK_GRAD, M, dY.device)
    wst = w.c_struct()
    _check(raw.qeft_linear_bwd(C.byref(desc), C.byref(wst), _ptr(dY), M, dY.stride(0) if M else desc.out_features, _ptr(dX),
                               dX.stride(0) if M else desc.in_features, _ptr(Xw), Xw.stride(0) if M else max(desc.n_weak, 8),
                               _ptr(dW), code, int(bool(accumulate)), _ptr(ws), ws.numel() if ws is not None else 0, _stream()),
           "qeft_linear_bwd")
    return dX, dW

