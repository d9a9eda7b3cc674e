"""Helpers shared by the GPU parity tests: build a stored layer on the device from host
arrays through the C-ABI, and the tolerance of the parity bar."""
import numpy as np
import torch

from oracle import qeft_oracle as qo
from paper_2410_08661_amd import binding as B
from paper_2410_08661_amd import synth

REL = 2e-3   # the stated bar: relative error <= 2e-3 with fp32 accumulation


def assert_close(actual, ref64, what=""):
    """Frobenius-relative error <= REL and, per element, |a - r| <= REL * (|r| + rms(r)).
    The rms floor keeps outputs that are near zero by cancellation from failing on noise
    that is small against the size of the terms that cancelled."""
    a = np.asarray(actual, dtype=np.float64)
    r = np.asarray(ref64, dtype=np.float64)
    assert a.shape == r.shape, (a.shape, r.shape)
    if r.size == 0:
        return
    assert np.all(np.isfinite(a)), f"{what}: non-finite output"
    rms = float(np.sqrt(np.mean(r * r)))
    fro = float(np.linalg.norm(a - r)) / max(float(np.linalg.norm(r)), 1e-300)
    worst = float(np.max(np.abs(a - r) - REL * (np.abs(r) + rms)))
    assert fro <= REL, f"{what}: relative Frobenius error {fro:.3e} > {REL}"
    assert worst <= 0, f"{what}: element error exceeds bar by {worst:.3e} (rms {rms:.3e})"


class HostLayer:
    """One layer as the oracle sees it (host arrays) plus its device twin."""

    def __init__(self, oc, ic, k, bits, g, seed, quantizer="codes", dense=False):
        self.oc, self.ic, self.k, self.bits, self.g = oc, ic, k, bits, g
        self.lay = qo.layout(oc, ic, k, bits, g, dense=dense)
        self.kq = self.lay["kq"]
        self.desc = B.make_desc(oc, ic, k, bits, g, layout=B.QEFT_LAYOUT_DENSE3 if dense else B.QEFT_LAYOUT_CANONICAL)
        w = synth.make_weight(oc, ic, seed)
        if quantizer == "rtn":
            self.codes, self.scales, self.zeros, self.weak = qo.quantize_rtn(w, k, bits, g)
        else:
            self.codes, self.scales, self.zeros = synth.make_codes(oc, self.kq, self.lay["n_groups"], bits, seed)
            self.weak = np.ascontiguousarray(w[:, ic - k:])
        if dense:
            self.qweight = qo.pack_codes_dense3(self.codes, self.lay["row_stride_words"])
        else:
            self.qweight = qo.pack_codes(self.codes, bits, self.lay["row_stride_words"])
        self._w64 = None

    @property
    def w64(self):
        if self._w64 is None:
            self._w64 = qo.dequantize(self.codes, self.scales, self.zeros, self.weak, self.g)
        return self._w64

    def to_device(self):
        """Upload the oracle-packed components as they are (no GPU packing involved)."""
        w = B.Weight(self.desc)
        if self.kq:
            w.qweight.copy_(torch.from_numpy(self.qweight.view(np.int32)))
            ng = self.lay["n_groups"]            # stored rows are padded to group_stride with zeros
            w.scales[:, :ng].copy_(torch.from_numpy(self.scales))
            w.zeros[:, :ng].copy_(torch.from_numpy(self.zeros))
        if self.k:
            w.weak.copy_(torch.from_numpy(self.weak))
        return w


def pad_cols(a, mult=8):
    """Return (device tensor view [M][cols], backing tensor) with a leading dimension that
    is a multiple of `mult` elements."""
    m, c = a.shape
    ld = -(-max(c, 1) // mult) * mult
    buf = torch.zeros((m, ld), dtype=torch.float16, device="cuda")
    if c:
        buf[:, :c].copy_(torch.from_numpy(np.ascontiguousarray(a)))
    return buf[:, :c], buf


class BigLayer:
    def __init__(self, oc, ic, k, bits, seed):
        # bits "3d": 3-bit codes in the dense layout
        dense = bits == "3d"
        nbits = 3 if dense else bits
        self.oc, self.ic, self.k, self.bits, self.nbits, self.g = oc, ic, k, bits, nbits, 128
        self.lay = qo.layout(oc, ic, k, nbits, 128, dense=dense)
        self.kq = self.lay["kq"]
        codes, self.scales, self.zeros = synth.make_codes(oc, self.kq, self.lay["n_groups"], nbits, seed)
        if dense:
            self.qweight = qo.pack_codes_dense3(codes, self.lay["row_stride_words"])
        else:
            self.qweight = qo.pack_codes(codes, bits, self.lay["row_stride_words"])
        del codes
        self.weak = (np.random.default_rng(seed).standard_normal((oc, k), dtype=np.float32) * 0.02).astype(np.float16)
        self.desc = B.make_desc(oc, ic, k, nbits, 128, layout=B.QEFT_LAYOUT_DENSE3 if dense else B.QEFT_LAYOUT_CANONICAL)
        w = B.Weight(self.desc)
        ng = self.lay["n_groups"]
        w.qweight.copy_(torch.from_numpy(self.qweight.view(np.int32)))
        w.scales[:, :ng].copy_(torch.from_numpy(self.scales))
        w.zeros[:, :ng].copy_(torch.from_numpy(self.zeros))
        w.weak.copy_(torch.from_numpy(self.weak))
        self.dev = w
        self._w64 = None

    @property
    def w64(self):
        """The whole mixed weight in float64, from the PACKED words (the oracle's unpack, then its dequantize)."""
        if self._w64 is None:
            codes = qo.unpack_codes_dense3(self.qweight, self.kq) if self.bits == "3d" else qo.unpack_codes(self.qweight, self.kq, self.nbits)
            self._w64 = qo.dequantize(codes, self.scales, self.zeros, self.weak, self.g)
        return self._w64
