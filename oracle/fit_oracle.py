"""ctypes front end of the encode-side C oracle (fit_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libfit_oracle.so")
_lib = None


def build() -> str:
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
           os.path.join(_HERE, "fit_oracle.c"), "-o", _SO, "-lm"]
    subprocess.run(cmd, check=True)
    return _SO


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(os.path.join(_HERE, "fit_oracle.c")):
            build()
        L = C.CDLL(_SO)
        vp, i32, i64, dbl = C.c_void_p, C.c_int32, C.c_int64, C.c_double
        L.fit_n_params.argtypes = [vp, i32]; L.fit_n_params.restype = i64
        L.fit_loss_grad.argtypes = [vp, i32, dbl, dbl, dbl, i32, i32, vp, vp, vp, dbl, vp, vp]; L.fit_loss_grad.restype = None
        L.fit_forward.argtypes = [vp, i32, dbl, dbl, dbl, i32, i32, vp, vp, vp]; L.fit_forward.restype = None
        L.fit_adam_step.argtypes = [vp, vp, vp, vp, vp, i64, i32, dbl, dbl, dbl, dbl]; L.fit_adam_step.restype = None
        L.fit_cosine_lr.argtypes = [dbl, i32, i32]; L.fit_cosine_lr.restype = dbl
        L.fit_psnr.argtypes = [vp, vp, i64]; L.fit_psnr.restype = dbl
        L.fit_prune_ratio.argtypes = [i32, dbl]; L.fit_prune_ratio.restype = dbl
        L.fit_l1_mask.argtypes = [vp, i64, dbl, vp, vp]; L.fit_l1_mask.restype = None
        L.fit_quantize.argtypes = [vp, vp, i64, i32, vp, vp, vp]; L.fit_quantize.restype = None
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data


def _w(widths):
    return np.ascontiguousarray(widths, dtype=np.int32)


def n_params(widths) -> int:
    w = _w(widths)
    return int(lib().fit_n_params(_p(w), len(w) - 1))


def loss_grad(widths, params, target, keep=None, w0=30.0, lo=-1.0, hi=1.0, loss_scale=None, want_grad=True):
    """target [3, H, W]; returns (loss, grad or None)."""
    w = _w(widths)
    target = np.ascontiguousarray(target, dtype=np.float64)
    _, H, W = target.shape
    params = np.ascontiguousarray(params, dtype=np.float64)
    keep = None if keep is None else np.ascontiguousarray(keep, dtype=np.uint8)
    if loss_scale is None:
        loss_scale = 1.0 / target.size
    loss = C.c_double()
    grad = np.empty_like(params) if want_grad else None
    lib().fit_loss_grad(_p(w), len(w) - 1, w0, lo, hi, H, W, _p(params), _p(keep), _p(target), loss_scale,
                        C.addressof(loss), _p(grad))
    return loss.value, grad


def forward(widths, params, H, W, keep=None, w0=30.0, lo=-1.0, hi=1.0) -> np.ndarray:
    w = _w(widths)
    params = np.ascontiguousarray(params, dtype=np.float64)
    keep = None if keep is None else np.ascontiguousarray(keep, dtype=np.uint8)
    out = np.empty((int(w[-1]), H, W), dtype=np.float64)
    lib().fit_forward(_p(w), len(w) - 1, w0, lo, hi, H, W, _p(params), _p(keep), _p(out))
    return out


def adam_step(params, m, v, grad, t, lr, keep=None, b1=0.9, b2=0.999, eps=1e-8):
    """In place on params, m, v (float64 arrays)."""
    keep = None if keep is None else np.ascontiguousarray(keep, dtype=np.uint8)
    grad = np.ascontiguousarray(grad, dtype=np.float64)
    lib().fit_adam_step(_p(params), _p(m), _p(v), _p(grad), _p(keep), params.size, t, lr, b1, b2, eps)


def cosine_lr(lr0, t, T) -> float:
    return float(lib().fit_cosine_lr(lr0, t, T))


def psnr(a, b) -> float:
    a = np.ascontiguousarray(a, dtype=np.float64); b = np.ascontiguousarray(b, dtype=np.float64)
    return float(lib().fit_psnr(_p(a), _p(b), a.size))


def prune_ratio(schedule, psnr_db) -> float:
    return float(lib().fit_prune_ratio(schedule, psnr_db))


def l1_mask(w, ratio, keep_in=None) -> np.ndarray:
    w = np.ascontiguousarray(w, dtype=np.float64).ravel()
    keep_in = None if keep_in is None else np.ascontiguousarray(keep_in, dtype=np.uint8).ravel()
    out = np.empty(w.size, dtype=np.uint8)
    lib().fit_l1_mask(_p(w), w.size, ratio, _p(keep_in), _p(out))
    return out


def quantize(w, bits, keep=None):
    """Returns (scale, zp, codes uint16)."""
    w = np.ascontiguousarray(w, dtype=np.float64).ravel()
    keep = None if keep is None else np.ascontiguousarray(keep, dtype=np.uint8).ravel()
    scale, zp = C.c_double(), C.c_int32()
    codes = np.empty(w.size, dtype=np.uint16)
    lib().fit_quantize(_p(w), _p(keep), w.size, bits, C.addressof(scale), C.addressof(zp), _p(codes))
    return scale.value, zp.value, codes


def fit(widths, params0, target, steps, lr0, T=None, keep=None, w0=30.0, lo=-1.0, hi=1.0, loss_scale=None,
        b1=0.9, b2=0.999, eps=1e-8):
    """`steps` full-batch Adam steps with cosine decay over T (default: steps).  Returns (params, losses)."""
    p = np.array(params0, dtype=np.float64)
    if keep is not None:
        p = p * (np.asarray(keep) != 0)
    m, v = np.zeros_like(p), np.zeros_like(p)
    T = steps if T is None else T
    losses = []
    for t in range(steps):
        loss, g = loss_grad(widths, p, target, keep, w0, lo, hi, loss_scale)
        losses.append(loss)
        adam_step(p, m, v, g, t + 1, cosine_lr(lr0, t, T), keep, b1, b2, eps)
    return p, losses
