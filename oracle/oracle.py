"""ctypes front end of the C oracle (inr_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this.
Models are duck-typed: an object with `.layers`, each layer having n_in, n_out,
bits, scale, zp, weights ([n_out, n_in] float32 or integer codes), keep (None or
[n_out, n_in] of 0/1) and bias ([n_out] float32).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libinr_oracle.so")


class _Layer(C.Structure):
    _fields_ = [("n_in", C.c_int32), ("n_out", C.c_int32), ("bits", C.c_int32), ("zp", C.c_int32),
                ("scale", C.c_float), ("w_f32", C.c_void_p), ("codes", C.c_void_p),
                ("keep", C.c_void_p), ("bias", C.c_void_p)]


class _Model(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("layers", C.POINTER(_Layer))]


def build() -> str:
    """Compile the C oracle with gcc (ISO C, no fast-math, OpenMP over images)."""
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           os.path.join(_HERE, "inr_oracle.c"), "-o", _SO, "-lm"]
    subprocess.run(cmd, check=True)
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        L = C.CDLL(_SO)
        L.orc_dequant.argtypes = [C.POINTER(_Layer), C.c_void_p]
        L.orc_dequant.restype = None
        L.orc_decode.argtypes = [C.POINTER(_Model), C.c_int64, C.c_void_p, C.c_int64, C.c_int32, C.c_int32,
                                 C.c_double, C.c_double, C.c_double, C.c_int, C.c_void_p, C.c_void_p, C.c_int]
        L.orc_decode.restype = C.c_int
        L.orc_decode_aug.argtypes = [C.POINTER(_Model), C.c_int64, C.c_void_p, C.c_int64, C.c_int32, C.c_int32,
                                     C.c_double, C.c_double, C.c_double, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]
        L.orc_decode_aug.restype = C.c_int
        _lib = L
    return _lib


def _marshal_layer(ly, hold):
    s = _Layer()
    s.n_in, s.n_out, s.bits, s.zp = int(ly.n_in), int(ly.n_out), int(ly.bits), int(ly.zp)
    s.scale = float(ly.scale)
    if ly.bits == 0:
        w = np.ascontiguousarray(ly.weights, dtype=np.float32).reshape(-1)
        s.w_f32, s.codes = w.ctypes.data, None
    else:
        w = np.ascontiguousarray(ly.weights).astype(np.uint16).reshape(-1)
        s.w_f32, s.codes = None, w.ctypes.data
    hold.append(w)
    if ly.keep is None:
        s.keep = None
    else:
        k = np.ascontiguousarray(ly.keep, dtype=np.uint8).reshape(-1)
        hold.append(k)
        s.keep = k.ctypes.data
    b = np.ascontiguousarray(ly.bias, dtype=np.float32).reshape(-1)
    hold.append(b)
    s.bias = b.ctypes.data
    assert w.size == ly.n_in * ly.n_out and b.size == ly.n_out
    return s


def dequant(layer) -> np.ndarray:
    """Effective weights [n_out, n_in] of one layer (float64 holding fp32 values)."""
    hold = []
    s = _marshal_layer(layer, hold)
    out = np.empty(layer.n_in * layer.n_out, dtype=np.float64)
    lib().orc_dequant(C.byref(s), out.ctypes.data)
    return out.reshape(layer.n_out, layer.n_in)


def decode(models, image_ids, H, W, w0=30.0, lo=-1.0, hi=1.0, clamp=True, want_u8=False, n_threads=None,
           affine=None, norm=None):
    """Decode slots; only the models that image_ids names are marshalled.

    Returns out_f64 [n, 3, H, W] (and out_u8 of the same shape when want_u8).
    affine: None or [n, 6] per-slot map of the sampling grid; norm: None or (scale[3], shift[3]).
    """
    ids = np.ascontiguousarray(image_ids, dtype=np.int64)
    n = len(ids)
    if n_threads is None:
        n_threads = os.cpu_count() or 1
    uniq, inv = np.unique(ids, return_inverse=True) if n else (np.zeros(0, np.int64), np.zeros(0, np.int64))
    if n and (uniq[0] < 0 or uniq[-1] >= len(models)):
        raise ValueError("image id out of range")
    hold = []
    arr = (_Model * max(1, len(uniq)))()
    for j, mid in enumerate(uniq):
        m = models[int(mid)]
        la = (_Layer * len(m.layers))(*[_marshal_layer(ly, hold) for ly in m.layers])
        hold.append(la)
        arr[j].n_layers = len(m.layers)
        arr[j].layers = la
    local_ids = np.ascontiguousarray(inv, dtype=np.int64)
    out = np.empty((n, 3, H, W), dtype=np.float64)
    out8 = np.empty((n, 3, H, W), dtype=np.uint8) if want_u8 else None
    if affine is not None or norm is not None:
        if want_u8:
            raise ValueError("uint8 output is not defined with augmentation")
        aff = None if affine is None else np.ascontiguousarray(affine, dtype=np.float64).reshape(n, 6)
        nrm = None if norm is None else np.ascontiguousarray(np.concatenate([norm[0], norm[1]]), dtype=np.float64)
        rc = lib().orc_decode_aug(arr, len(uniq), local_ids.ctypes.data, n, H, W, float(w0), float(lo), float(hi),
                                  1 if clamp else 0, None if aff is None else aff.ctypes.data,
                                  None if nrm is None else nrm.ctypes.data, out.ctypes.data, int(n_threads))
    else:
        rc = lib().orc_decode(arr, len(uniq), local_ids.ctypes.data, n, H, W, float(w0), float(lo), float(hi),
                              1 if clamp else 0, out.ctypes.data, out8.ctypes.data if want_u8 else None,
                              int(n_threads))
    if rc != 0:
        raise ValueError("orc_decode rejected its arguments")
    return (out, out8) if want_u8 else out
