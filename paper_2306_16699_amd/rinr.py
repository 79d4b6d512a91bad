"""ctypes binding of the rinr C ABI (include/rinr.h): argument marshalling only.

Every step of the decode runs in the HIP library.  PyTorch appears here only as the
owner of device memory and streams.  There is no fallback: if `librinr.so` has not
been built, `lib()` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SO_PATH = os.path.join(_HERE, "librinr.so")

OK = 0
OUT_F32, OUT_U8, OUT_F32_AND_U8 = 1, 2, 3
FLAG_NO_CLAMP = 1
FLAG_FP32_MFMA = 2
FLAG_NORMALIZE = 4
FLAG_FP16_ACT = 8
FLAG_FP16_ALL = 16
FLAG_FP16_UNCHECKED = 32
FAMILIES = ("split precision (fp16 hi+lo pairs)", "fp32 MFMA", "fp16 activations", "fp16 weights and activations")
E_NULL, E_ARG, E_MODEL, E_SIZE, E_FORMAT, E_UNSUPPORTED, E_ALIGN, E_HIP = -1, -2, -3, -4, -5, -6, -7, -8

EXPORTS = ["rinr_pack_size", "rinr_pack", "rinr_unpack_layer", "rinr_store_open", "rinr_store_open_ex", "rinr_store_close",
           "rinr_store_info", "rinr_store_error_bounds", "rinr_decode_batch", "rinr_decode_batch_ex", "rinr_decode_batch_noalloc", "rinr_store_status",
           "rinr_debug_dequant", "rinr_debug_dequant_split", "rinr_last_launch_info", "rinr_strerror",
           "rinr_last_hip_error", "rinr_version", "rinr_decode_workspace_bytes"]


class LayerDesc(C.Structure):
    _fields_ = [("n_in", C.c_int32), ("n_out", C.c_int32), ("bits", C.c_int32), ("scale", C.c_float),
                ("zp", C.c_int32), ("weights", C.c_void_p), ("mask", C.c_void_p), ("bias", C.c_void_p)]


class ModelDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("layers", C.POINTER(LayerDesc))]


class StoreOpts(C.Structure):
    _fields_ = [("w0", C.c_float), ("coord_lo", C.c_float), ("coord_hi", C.c_float)]


class OpenOpts(C.Structure):
    _fields_ = [("fp32_tile_rows", C.c_int32), ("lds_budget", C.c_int32)]


class DecodeOpts(C.Structure):
    _fields_ = [("out_dtype", C.c_int32), ("flags", C.c_int32), ("out_u8", C.c_void_p), ("affine", C.c_void_p),
                ("norm_scale", C.c_float * 3), ("norm_shift", C.c_float * 3), ("workspace", C.c_void_p),
                ("workspace_bytes", C.c_size_t), ("launch_threads", C.c_int32), ("launch_blocks_per_cu", C.c_int32),
                ("one_grid_min_tiles", C.c_int32)]


class RinrError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} ({code})")


_lib = None


def lib():
    """Loads librinr.so; raises if it is missing (build with `python -m paper_2306_16699_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(SO_PATH):
            raise FileNotFoundError(f"{SO_PATH} not built; run python -m paper_2306_16699_amd.build")
        L = C.CDLL(SO_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.rinr_pack_size.argtypes = [C.POINTER(ModelDesc), i64, C.POINTER(StoreOpts), C.POINTER(C.c_size_t)]
        L.rinr_pack.argtypes = [C.POINTER(ModelDesc), i64, C.POINTER(StoreOpts), vp, C.c_size_t]
        L.rinr_unpack_layer.argtypes = [vp, C.c_size_t, i64, i32, vp, vp, vp, vp, C.POINTER(i32 * 5), C.POINTER(C.c_float)]
        L.rinr_store_open.argtypes = [vp, vp, C.c_size_t, C.POINTER(vp)]
        L.rinr_store_open_ex.argtypes = [vp, vp, C.c_size_t, C.POINTER(OpenOpts), C.POINTER(vp)]
        L.rinr_store_error_bounds.argtypes = [vp, C.POINTER(C.c_float * 2)]
        L.rinr_store_close.argtypes = [vp]
        L.rinr_store_info.argtypes = [vp, C.POINTER(i64), C.POINTER(i32), C.POINTER(i32)]
        L.rinr_decode_batch.argtypes = [vp, vp, i32, i32, i32, vp, vp]
        L.rinr_decode_batch_ex.argtypes = [vp, vp, i32, i32, i32, vp, C.POINTER(DecodeOpts), vp]
        L.rinr_decode_batch_noalloc.argtypes = [vp, vp, i32, i32, i32, vp, C.POINTER(DecodeOpts), vp]
        L.rinr_store_status.argtypes = [vp, C.POINTER(i64), vp]
        L.rinr_debug_dequant.argtypes = [vp, i64, i32, vp, vp, vp]
        L.rinr_debug_dequant_split.argtypes = [vp, i64, i32, i32, vp, vp, vp, vp, vp]
        L.rinr_last_launch_info.argtypes = [vp, C.POINTER(i32 * 6)]
        L.rinr_strerror.argtypes = [C.c_int]
        L.rinr_strerror.restype = C.c_char_p
        L.rinr_version.restype = C.c_char_p
        for name in EXPORTS:
            if name not in ("rinr_strerror", "rinr_version"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().rinr_strerror(code).decode()


def _check(rc: int, what: str):
    if rc != OK:
        raise RinrError(rc, what)


def workspace_bytes(n: int) -> int:
    L = lib()
    L.rinr_decode_workspace_bytes.restype = C.c_size_t
    L.rinr_decode_workspace_bytes.argtypes = [C.c_int32]
    return int(L.rinr_decode_workspace_bytes(n))


def pack_mask(keep: np.ndarray) -> np.ndarray:
    """0/1 per weight, flat index o*in + i -> bytes, bit k%8 of byte k/8."""
    return np.packbits(np.ascontiguousarray(keep, dtype=np.uint8).reshape(-1), bitorder="little")


def marshal_models(models: Sequence):
    """Model objects (see synth.Model) -> (ModelDesc array, keep-alive list)."""
    hold = []
    n_layers_total = sum(len(m.layers) for m in models)
    layers = (LayerDesc * max(1, n_layers_total))()
    descs = (ModelDesc * max(1, len(models)))()
    base = C.addressof(layers)
    k = 0
    for j, m in enumerate(models):
        descs[j].n_layers = len(m.layers)
        descs[j].layers = C.cast(base + k * C.sizeof(LayerDesc), C.POINTER(LayerDesc))
        for ly in m.layers:
            d = layers[k]
            k += 1
            d.n_in, d.n_out, d.bits, d.zp = int(ly.n_in), int(ly.n_out), int(ly.bits), int(ly.zp)
            d.scale = float(ly.scale)
            if ly.bits == 0:
                w = np.ascontiguousarray(ly.weights, dtype=np.float32)
            elif ly.bits <= 8:
                w = np.ascontiguousarray(ly.weights, dtype=np.uint8)
            else:
                w = np.ascontiguousarray(ly.weights, dtype=np.uint16)
            b = np.ascontiguousarray(ly.bias, dtype=np.float32)
            hold.append(w)
            hold.append(b)
            d.weights, d.bias = w.ctypes.data, b.ctypes.data
            if ly.keep is None:
                d.mask = None
            else:
                mk = pack_mask(ly.keep)
                hold.append(mk)
                d.mask = mk.ctypes.data
    hold.append(layers)
    return descs, hold


def pack(models: Sequence, w0: float = 30.0, coord_lo: float = -1.0, coord_hi: float = 1.0) -> np.ndarray:
    """rinr_pack_size + rinr_pack: returns the blob as a uint8 array (host)."""
    descs, hold = marshal_models(models)
    opts = StoreOpts(w0, coord_lo, coord_hi)
    size = C.c_size_t(0)
    _check(lib().rinr_pack_size(descs, len(models), C.byref(opts), C.byref(size)), "rinr_pack_size")
    blob = np.zeros(size.value, dtype=np.uint8)
    _check(lib().rinr_pack(descs, len(models), C.byref(opts), blob.ctypes.data, size.value), "rinr_pack")
    del hold
    return blob


def unpack_layer(blob: np.ndarray, model: int, layer: int):
    """rinr_unpack_layer: dict(in, out, bits, zp, n_kept, scale, codes, f32, keep, bias)."""
    L = lib()
    meta = (C.c_int32 * 5)()
    scale = C.c_float(0)
    _check(L.rinr_unpack_layer(blob.ctypes.data, blob.size, model, layer, None, None, None, None,
                               C.byref(meta), C.byref(scale)), "rinr_unpack_layer")
    n_in, n_out = meta[0], meta[1]
    codes = np.zeros(n_in * n_out, np.uint16)
    f32 = np.zeros(n_in * n_out, np.float32)
    keep = np.zeros(n_in * n_out, np.uint8)
    bias = np.zeros(n_out, np.float32)
    _check(L.rinr_unpack_layer(blob.ctypes.data, blob.size, model, layer, codes.ctypes.data, f32.ctypes.data,
                               keep.ctypes.data, bias.ctypes.data, C.byref(meta), C.byref(scale)), "rinr_unpack_layer")
    return dict(n_in=n_in, n_out=n_out, bits=meta[2], zp=meta[3], n_kept=meta[4], scale=scale.value,
                codes=codes.reshape(n_out, n_in), f32=f32.reshape(n_out, n_in), keep=keep.reshape(n_out, n_in), bias=bias)


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


class Store:
    """A device-resident dataset in weight format.  Holds the device blob (a torch uint8 tensor)."""

    def __init__(self, blob: np.ndarray, device="cuda:0", validate_on_device: bool = False, fp32_tile_rows: int = 0,
                 lds_budget: int = 0):
        import torch
        self._torch = torch
        self.device = torch.device(device)
        self.host_blob = blob
        with torch.cuda.device(self.device):
            self.dev_blob = torch.from_numpy(blob).to(self.device)
            h = C.c_void_p(0)
            host = None if validate_on_device else blob.ctypes.data
            if fp32_tile_rows or lds_budget:
                oo = OpenOpts(fp32_tile_rows, lds_budget)
                _check(lib().rinr_store_open_ex(self.dev_blob.data_ptr(), host, blob.size, C.byref(oo), C.byref(h)), "rinr_store_open_ex")
            else:
                _check(lib().rinr_store_open(self.dev_blob.data_ptr(), host, blob.size, C.byref(h)), "rinr_store_open")
        self._h = h

    def close(self):
        if self._h:
            _check(lib().rinr_store_close(self._h), "rinr_store_close")
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def info(self):
        n, w, l = C.c_int64(0), C.c_int32(0), C.c_int32(0)
        _check(lib().rinr_store_info(self._h, C.byref(n), C.byref(w), C.byref(l)), "rinr_store_info")
        return n.value, w.value, l.value

    def error_bounds(self):
        """rinr_store_error_bounds: a-priori error bounds of FLAG_FP16_ACT and FLAG_FP16_ALL on this store."""
        b = (C.c_float * 2)()
        _check(lib().rinr_store_error_bounds(self._h, C.byref(b)), "rinr_store_error_bounds")
        return float(b[0]), float(b[1])

    def decode_batch(self, image_ids, H: int, W: int, out=None, stream=None):
        """rinr_decode_batch: fp32 NCHW, clamped to [0, 1].  image_ids: int64 CUDA tensor."""
        torch = self._torch
        n = int(image_ids.numel())
        if out is None:
            out = torch.empty((n, 3, H, W), dtype=torch.float32, device=self.device)
        _check(lib().rinr_decode_batch(self._h, image_ids.data_ptr() if n else None, n, H, W,
                                       out.data_ptr() if n else None, _stream_ptr(stream)), "rinr_decode_batch")
        return out

    def decode_batch_ex(self, image_ids, H: int, W: int, out_dtype: int = OUT_F32, flags: int = 0,
                        out=None, out_u8=None, stream=None, affine=None, norm=None, workspace=None,
                        threads: int = 0, blocks_per_cu: int = 0, one_grid_min_tiles: int = 0, noalloc: bool = False):
        """rinr_decode_batch_ex.  Returns out (and out_u8 for OUT_F32_AND_U8).

        workspace: uint8 CUDA tensor of >= workspace_bytes(n) bytes (heaviest-first order for ragged stores) or None;

        affine: float32 CUDA tensor [n, 6] (per-slot map of the sampling grid) or None;
        norm: (scale[3], shift[3]) host numbers, sets FLAG_NORMALIZE;
        threads, blocks_per_cu, one_grid_min_tiles: launch shape (0 = the library's choice);
        noalloc: call rinr_decode_batch_noalloc (slot order in the library's static scratch) instead."""
        torch = self._torch
        n = int(image_ids.numel())
        if out is None:
            out = torch.empty((n, 3, H, W), dtype=torch.uint8 if out_dtype == OUT_U8 else torch.float32,
                              device=self.device)
        if out_dtype == OUT_F32_AND_U8 and out_u8 is None:
            out_u8 = torch.empty((n, 3, H, W), dtype=torch.uint8, device=self.device)
        o = DecodeOpts(out_dtype, flags, out_u8.data_ptr() if (out_u8 is not None and n) else None)
        o.launch_threads, o.launch_blocks_per_cu, o.one_grid_min_tiles = threads, blocks_per_cu, one_grid_min_tiles
        if affine is not None:
            assert affine.dtype == torch.float32 and affine.is_contiguous() and tuple(affine.shape) == (n, 6)
            o.affine = affine.data_ptr() if n else None
        if workspace is not None and n:
            assert workspace.is_cuda and workspace.dtype == torch.uint8 and workspace.is_contiguous()
            o.workspace, o.workspace_bytes = workspace.data_ptr(), workspace.numel()
        if norm is not None:
            o.flags |= FLAG_NORMALIZE
            o.norm_scale = (C.c_float * 3)(*[float(v) for v in norm[0]])
            o.norm_shift = (C.c_float * 3)(*[float(v) for v in norm[1]])
        fn = lib().rinr_decode_batch_noalloc if noalloc else lib().rinr_decode_batch_ex
        _check(fn(self._h, image_ids.data_ptr() if n else None, n, H, W, out.data_ptr() if n else None, C.byref(o),
                  _stream_ptr(stream)), "rinr_decode_batch_noalloc" if noalloc else "rinr_decode_batch_ex")
        return (out, out_u8) if out_dtype == OUT_F32_AND_U8 else out

    def status(self, stream=None) -> int:
        v = C.c_int64(0)
        _check(lib().rinr_store_status(self._h, C.byref(v), _stream_ptr(stream)), "rinr_store_status")
        return v.value

    def debug_dequant(self, model: int, layer: int, n_in: int, n_out: int, stream=None):
        torch = self._torch
        w = torch.empty((n_out, n_in), dtype=torch.float32, device=self.device)
        b = torch.empty((n_out,), dtype=torch.float32, device=self.device)
        _check(lib().rinr_debug_dequant(self._h, model, layer, w.data_ptr(), b.data_ptr(), _stream_ptr(stream)),
               "rinr_debug_dequant")
        return w, b

    def debug_dequant_split(self, model: int, layer: int, n_in: int, n_out: int, fp16_weights: bool = False, stream=None):
        """rinr_debug_dequant_split: (hi, lo, bias, scale) of the split-precision kernels' operand blocks."""
        torch = self._torch
        hi = torch.empty((n_out, n_in), dtype=torch.float32, device=self.device)
        lo = torch.empty((n_out, n_in), dtype=torch.float32, device=self.device)
        b = torch.empty((n_out,), dtype=torch.float32, device=self.device)
        sc = torch.empty((1,), dtype=torch.float32, device=self.device)
        _check(lib().rinr_debug_dequant_split(self._h, model, layer, 1 if fp16_weights else 0, hi.data_ptr(), lo.data_ptr(),
                                              b.data_ptr(), sc.data_ptr(), _stream_ptr(stream)), "rinr_debug_dequant_split")
        return hi, lo, b, sc

    def last_launch_info(self):
        info = (C.c_int32 * 6)()
        _check(lib().rinr_last_launch_info(self._h, C.byref(info)), "rinr_last_launch_info")
        return dict(launches=info[0], workgroups=info[1], threads=info[2], lds_bytes=info[3], kernels=FAMILIES[info[4]],
                    streamed=bool(info[5]))
