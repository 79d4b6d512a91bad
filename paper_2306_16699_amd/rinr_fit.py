"""ctypes binding of include/rinr_fit.h (the encode side): argument marshalling only.

Fitting runs in the HIP kernels of librinr.so; pruning-ratio schedule, magnitude masks and the
quantiser are the library's host functions.  PyTorch is used for device memory and streams.
"""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence

import numpy as np

from . import rinr
from .synth import Layer, Model

MAX_LAYERS = 12
FIT_FLAG_FP32_MFMA = 1
KERNEL_FP32, KERNEL_SPLIT16 = 0, 1
EXPORTS = ["rinr_prune_ratio", "rinr_l1_mask", "rinr_quantize_layer", "rinr_fit_create", "rinr_fit_create_ex", "rinr_fit_kernel_family",
           "rinr_fit_destroy",
           "rinr_fit_n_params", "rinr_fit_set_params", "rinr_fit_set_keep", "rinr_fit_reset_optimizer",
           "rinr_fit_get_params", "rinr_fit_steps", "rinr_fit_loss_grad", "rinr_fit_last_loss", "rinr_psnr_batch", "rinr_encode_blob_bound",
           "rinr_encode_images"]


class FitArch(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("widths", C.c_int32 * (MAX_LAYERS + 1)), ("w0", C.c_float),
                ("coord_lo", C.c_float), ("coord_hi", C.c_float)]


class FitOpts(C.Structure):
    _fields_ = [("lr", C.c_float), ("t0", C.c_int32), ("T", C.c_int32), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("loss_scale", C.c_float)]


class EncodeOpts(C.Structure):
    _fields_ = [("schedule", C.c_int32), ("first_ratio", C.c_float), ("fit_steps", C.c_int32), ("refit_steps", C.c_int32),
                ("lr", C.c_float), ("refit_lr", C.c_float), ("hidden_bits", C.c_int32)]


_ready = False


def lib():
    global _ready
    L = rinr.lib()
    if not _ready:
        vp, i32, i64, dbl = C.c_void_p, C.c_int32, C.c_int64, C.c_double
        L.rinr_prune_ratio.argtypes = [i32, dbl]
        L.rinr_prune_ratio.restype = dbl
        L.rinr_l1_mask.argtypes = [vp, i64, dbl, vp, vp]
        L.rinr_quantize_layer.argtypes = [vp, vp, i64, i32, C.POINTER(C.c_float), C.POINTER(i32), vp]
        L.rinr_fit_create.argtypes = [C.POINTER(FitArch), i64, i32, i32, C.POINTER(vp)]
        L.rinr_fit_create_ex.argtypes = [C.POINTER(FitArch), i64, i32, i32, C.c_uint32, C.POINTER(vp)]
        L.rinr_fit_kernel_family.argtypes = [vp]
        L.rinr_fit_destroy.argtypes = [vp]
        L.rinr_fit_n_params.argtypes = [vp]
        L.rinr_fit_n_params.restype = i64
        L.rinr_fit_set_params.argtypes = [vp, vp]
        L.rinr_fit_set_keep.argtypes = [vp, vp]
        L.rinr_fit_reset_optimizer.argtypes = [vp]
        L.rinr_fit_get_params.argtypes = [vp, vp, vp]
        L.rinr_fit_steps.argtypes = [vp, vp, i32, C.POINTER(FitOpts), vp]
        L.rinr_fit_loss_grad.argtypes = [vp, vp, C.c_float, vp, vp, vp]
        L.rinr_fit_last_loss.argtypes = [vp, vp, vp]
        L.rinr_psnr_batch.argtypes = [vp, vp, i64, i64, C.c_float, vp, vp]
        L.rinr_encode_blob_bound.argtypes = [vp, i32, C.POINTER(C.c_size_t)]
        L.rinr_encode_images.argtypes = [vp, vp, C.POINTER(EncodeOpts), vp, vp, C.c_size_t, C.POINTER(C.c_size_t), vp]
        _ready = True
    return L


def prune_ratio(schedule: int, psnr: float) -> float:
    return float(lib().rinr_prune_ratio(schedule, psnr))


def l1_mask(w: np.ndarray, ratio: float, keep_in: Optional[np.ndarray] = None) -> np.ndarray:
    w = np.ascontiguousarray(w, dtype=np.float32).ravel()
    keep_in = None if keep_in is None else np.ascontiguousarray(keep_in, dtype=np.uint8).ravel()
    out = np.empty(w.size, dtype=np.uint8)
    rinr._check(lib().rinr_l1_mask(w.ctypes.data, w.size, ratio, None if keep_in is None else keep_in.ctypes.data,
                                   out.ctypes.data), "rinr_l1_mask")
    return out


def quantize_layer(w: np.ndarray, bits: int, keep: Optional[np.ndarray] = None):
    """Returns (scale float32, zp int, codes uint16[n])."""
    w = np.ascontiguousarray(w, dtype=np.float32).ravel()
    keep = None if keep is None else np.ascontiguousarray(keep, dtype=np.uint8).ravel()
    scale, zp = C.c_float(), C.c_int32()
    codes = np.empty(w.size, dtype=np.uint16)
    rinr._check(lib().rinr_quantize_layer(w.ctypes.data, None if keep is None else keep.ctypes.data, w.size, bits,
                                          C.byref(scale), C.byref(zp), codes.ctypes.data), "rinr_quantize_layer")
    return np.float32(scale.value), int(zp.value), codes


def psnr_batch(a, b, peak: float = 1.0, stream=None):
    """PSNR in dB per image of two device float32 tensors [n, ...] (torch); returns a device tensor [n]."""
    import torch
    assert a.is_cuda and b.is_cuda and a.dtype == torch.float32 and b.dtype == torch.float32
    assert a.shape == b.shape and a.is_contiguous() and b.is_contiguous()
    n = a.shape[0]
    out = torch.empty((n,), dtype=torch.float32, device=a.device)
    elems = a.numel() // n if n else 0
    rinr._check(lib().rinr_psnr_batch(a.data_ptr(), b.data_ptr(), n, elems, peak, out.data_ptr(), rinr._stream_ptr(stream)),
                "rinr_psnr_batch")
    return out


class Fit:
    """Device state for fitting n_images models of one architecture (widths = [2, ..., 3])."""

    def __init__(self, widths: Sequence[int], n_images: int, H: int, W: int, w0: float = 30.0,
                 coord_lo: float = -1.0, coord_hi: float = 1.0, fp32: bool = False):
        self.widths = [int(x) for x in widths]
        if len(self.widths) - 1 > MAX_LAYERS:
            raise rinr.RinrError(rinr.E_ARG, "rinr_fit_create")
        arch = FitArch()
        arch.n_layers = len(self.widths) - 1
        for i, x in enumerate(self.widths):
            arch.widths[i] = x
        arch.w0, arch.coord_lo, arch.coord_hi = w0, coord_lo, coord_hi
        self.w0, self.coord_lo, self.coord_hi = w0, coord_lo, coord_hi
        self.n_images, self.H, self.W = n_images, H, W
        h = C.c_void_p()
        rinr._check(lib().rinr_fit_create_ex(C.byref(arch), n_images, H, W, FIT_FLAG_FP32_MFMA if fp32 else 0, C.byref(h)),
                    "rinr_fit_create_ex")
        self._h = h
        self.kernel_family = int(lib().rinr_fit_kernel_family(h))      # KERNEL_FP32 or KERNEL_SPLIT16
        self.n_params = int(lib().rinr_fit_n_params(h))

    def close(self):
        if getattr(self, "_h", None):
            lib().rinr_fit_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_params(self, params: np.ndarray):
        p = np.ascontiguousarray(params, dtype=np.float32)
        assert p.shape == (self.n_images, self.n_params), p.shape
        rinr._check(lib().rinr_fit_set_params(self._h, p.ctypes.data), "rinr_fit_set_params")

    def set_keep(self, keep: Optional[np.ndarray]):
        if keep is None:
            rinr._check(lib().rinr_fit_set_keep(self._h, None), "rinr_fit_set_keep")
            return
        k = np.ascontiguousarray(keep, dtype=np.uint8)
        assert k.shape == (self.n_images, self.n_params), k.shape
        rinr._check(lib().rinr_fit_set_keep(self._h, k.ctypes.data), "rinr_fit_set_keep")

    def reset_optimizer(self):
        rinr._check(lib().rinr_fit_reset_optimizer(self._h), "rinr_fit_reset_optimizer")

    def get_params(self, stream=None) -> np.ndarray:
        out = np.empty((self.n_images, self.n_params), dtype=np.float32)
        rinr._check(lib().rinr_fit_get_params(self._h, out.ctypes.data, rinr._stream_ptr(stream)), "rinr_fit_get_params")
        return out

    def _targets(self, targets):
        import torch
        assert targets.is_cuda and targets.dtype == torch.float32 and targets.is_contiguous()
        assert tuple(targets.shape) == (self.n_images, 3, self.H, self.W), tuple(targets.shape)
        return targets.data_ptr()

    def steps(self, targets, n_steps: int, lr: float, t0: int = 0, T: int = 0, beta1: float = 0.0, beta2: float = 0.0,
              eps: float = 0.0, loss_scale: float = 0.0, stream=None):
        o = FitOpts(lr, t0, T, beta1, beta2, eps, loss_scale)
        rinr._check(lib().rinr_fit_steps(self._h, self._targets(targets), n_steps, C.byref(o), rinr._stream_ptr(stream)),
                    "rinr_fit_steps")

    def loss_grad(self, targets, loss_scale: float = 0.0, want_grad: bool = True, stream=None):
        loss = np.empty(self.n_images, dtype=np.float32)
        grad = np.empty((self.n_images, self.n_params), dtype=np.float32) if want_grad else None
        rinr._check(lib().rinr_fit_loss_grad(self._h, self._targets(targets), loss_scale, loss.ctypes.data,
                                             None if grad is None else grad.ctypes.data, rinr._stream_ptr(stream)),
                    "rinr_fit_loss_grad")
        return loss, grad

    def encode(self, targets, schedule: int, first_ratio: float, fit_steps: int, refit_steps: int, lr: float, refit_lr: float,
               hidden_bits: int = 8, stream=None):
        """rinr_encode_images: returns (blob uint8 array, psnr float32[n_images])."""
        bound = C.c_size_t()
        rinr._check(lib().rinr_encode_blob_bound(self._h, hidden_bits, C.byref(bound)), "rinr_encode_blob_bound")
        blob = np.empty(bound.value, dtype=np.uint8)
        psnr = np.empty(self.n_images, dtype=np.float32)
        o = EncodeOpts(schedule, first_ratio, fit_steps, refit_steps, lr, refit_lr, hidden_bits)
        size = C.c_size_t()
        rinr._check(lib().rinr_encode_images(self._h, self._targets(targets), C.byref(o), psnr.ctypes.data, blob.ctypes.data,
                                             bound.value, C.byref(size), rinr._stream_ptr(stream)), "rinr_encode_images")
        return blob[:size.value], psnr

    def last_loss(self, stream=None) -> np.ndarray:
        loss = np.empty(self.n_images, dtype=np.float32)
        rinr._check(lib().rinr_fit_last_loss(self._h, loss.ctypes.data, rinr._stream_ptr(stream)), "rinr_fit_last_loss")
        return loss


def split_params(widths: Sequence[int], params: np.ndarray):
    """One image's parameter vector -> [(W [out, in], b [out]) per layer] (views)."""
    out, off = [], 0
    for l in range(len(widths) - 1):
        nin, nout = widths[l], widths[l + 1]
        w = params[off:off + nout * nin].reshape(nout, nin)
        off += nout * nin
        out.append((w, params[off:off + nout]))
        off += nout
    return out


def weight_keep_flags(widths: Sequence[int], keep_mats: List[Optional[np.ndarray]]) -> np.ndarray:
    """Per-parameter keep flags from per-matrix flags (biases are always kept)."""
    parts = []
    for l in range(len(widths) - 1):
        nin, nout = widths[l], widths[l + 1]
        k = keep_mats[l]
        parts.append(np.ones(nout * nin, np.uint8) if k is None else np.asarray(k, np.uint8).ravel())
        parts.append(np.ones(nout, np.uint8))
    return np.concatenate(parts)


def to_model(widths: Sequence[int], params: np.ndarray, keep_mats: Optional[List[Optional[np.ndarray]]] = None,
             hidden_bits: int = 8) -> Model:
    """Fitted parameters -> the model description rinr.pack takes: hidden layers as `hidden_bits`-bit
    codes from rinr_quantize_layer, first and last layer fp32 (Sec. IV-B); hidden_bits = 0 keeps all fp32."""
    layers = []
    L = len(widths) - 1
    for l, (w, b) in enumerate(split_params(widths, np.asarray(params, np.float32))):
        k = None if keep_mats is None or keep_mats[l] is None else np.asarray(keep_mats[l], np.uint8).reshape(w.shape)
        if hidden_bits and 0 < l < L - 1:
            scale, zp, codes = quantize_layer(w, hidden_bits, k)
            cw = codes.reshape(w.shape).astype(np.uint8 if hidden_bits <= 8 else np.uint16)
            layers.append(Layer(w.shape[1], w.shape[0], hidden_bits, scale, zp, cw, k, b.astype(np.float32).copy()))
        else:
            layers.append(Layer(w.shape[1], w.shape[0], 0, np.float32(1.0), 0, w.astype(np.float32).copy(), k,
                                b.astype(np.float32).copy()))
    return Model(layers)
