"""Seeded synthetic INR datasets (inputs only; none of the decode arithmetic).

Every image of the paper's dataset is its own small sine-activated MLP
(Sec. III-A), pruned with a mask (Sec. IV-A) and with hidden layers stored as
8-bit codes while the first and last layer stay fp32 (Sec. IV-B).  The paper's
datasets and trained weights are not available, so this module draws models of
the same shape from a counter-based generator: every number is a pure function
of (seed, model id, layer, tensor kind, element index), so any one model of a
large pool can be regenerated alone and both the CPU oracle's tests and the GPU
path's tests see identical inputs.

This module is shared input plumbing: it holds no dequantisation, no MLP
evaluation and no packing.  The oracle and the HIP library each consume the
plain arrays produced here through their own marshalling.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)

KIND_WEIGHT = 0
KIND_BIAS = 1
KIND_ARCH = 2
KIND_IDS = 3


def _mix(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function on a uint64 array (wrapping arithmetic)."""
    with np.errstate(over="ignore"):
        z = (z + _GOLD)
        z = (z ^ (z >> np.uint64(30))) * _C1
        z = (z ^ (z >> np.uint64(27))) * _C2
        return z ^ (z >> np.uint64(31))


def stream_key(seed: int, model, layer: int, kind: int) -> np.ndarray:
    """Key of one random stream; `model` may be an int or an int array."""
    m = np.asarray(model, dtype=np.uint64)
    k = _mix(np.asarray(seed, dtype=np.uint64))
    k = _mix(k ^ m)
    k = _mix(k ^ np.uint64(layer * 8 + kind))
    return k


def stream_bits(key: np.ndarray, n: int) -> np.ndarray:
    """n 64-bit words per key: shape key.shape + (n,)."""
    idx = np.arange(n, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix(key[..., None] + idx * _GOLD)


def _unit24(bits: np.ndarray) -> np.ndarray:
    """24-bit uniform in (0,1) as float64, from the top bits of each word."""
    return ((bits >> np.uint64(40)).astype(np.float64) + 0.5) / float(1 << 24)


@dataclass
class Layer:
    n_in: int
    n_out: int
    bits: int                      # 0 = raw fp32 weights, else code width
    scale: float                   # fp32 value; w = scale * (q - zp)
    zp: int
    weights: np.ndarray            # [n_out, n_in] float32 (bits==0) or uint8/uint16 codes
    keep: Optional[np.ndarray]     # [n_out, n_in] uint8 0/1, or None = dense
    bias: np.ndarray               # [n_out] float32


@dataclass
class Model:
    layers: List[Layer]

    @property
    def width(self) -> int:
        return max(l.n_out for l in self.layers[:-1]) if len(self.layers) > 1 else 0

    @property
    def n_sine_layers(self) -> int:
        return len(self.layers) - 1


def c_hidden(width: int, w0: float = 30.0) -> float:
    return math.sqrt(6.0 / width) / w0


def make_models(seed: int, ids: np.ndarray, width: int, n_sine: int,
                layer_bits: Sequence[Sequence[int]], keep_prob,
                w0: float = 30.0, widths: Optional[Sequence[int]] = None) -> List[Model]:
    """Models `ids` (all of one architecture), drawn in bulk.

    The chain is 2 -> width (x n_sine sine layers) -> 3, i.e. n_sine + 1 linear
    layers.  `widths` overrides the uniform width with a per-sine-layer list
    (tapered shapes).  `layer_bits[l]` is an int array over the models (or a
    scalar) giving layer l's code width, 0 meaning raw fp32.  `keep_prob` is a
    scalar or per-model array; None or >= 1 means no mask is stored.

    Value recipe: layer 0 raw weights U(-1/2, 1/2); other raw weights
    U(+-sqrt(6/fan_in)/w0); codes uniform on [0, 2^b), zero point 2^(b-1),
    scale = 2*sqrt(6/fan_in)/w0/(2^b - 1); biases U(-0.1, 0.1).
    """
    ids = np.asarray(ids, dtype=np.int64)
    nm = len(ids)
    hid = list(widths) if widths is not None else [width] * n_sine
    dims = [2] + hid + [3]
    n_lin = len(dims) - 1
    models = [Model(layers=[]) for _ in range(nm)]
    dense = keep_prob is None
    kp = None if dense else np.broadcast_to(np.asarray(keep_prob, dtype=np.float64), (nm,))
    for l in range(n_lin):
        n_in, n_out = dims[l], dims[l + 1]
        cnt = n_in * n_out
        bits_l = np.broadcast_to(np.asarray(layer_bits[l], dtype=np.int64), (nm,))
        raw = stream_bits(stream_key(seed, ids, l, KIND_WEIGHT), cnt)
        u = _unit24(raw)
        c = 0.5 if l == 0 else c_hidden(n_in, w0)
        w_f32 = ((2.0 * u - 1.0) * c).astype(np.float32)
        # disjoint bit fields of each word: 40..63 float, 24..39 code, 0..23 mask
        if dense:
            keep_all = None
        else:
            low = (raw & np.uint64(0xFFFFFF)).astype(np.uint32)
            thr = np.floor(kp * float(1 << 24)).astype(np.uint32)
            keep_all = (low < thr[:, None]).astype(np.uint8)
        ub = _unit24(stream_bits(stream_key(seed, ids, l, KIND_BIAS), n_out))
        bias = ((2.0 * ub - 1.0) * 0.1).astype(np.float32)
        for j in range(nm):
            b = int(bits_l[j])
            if b == 0:
                wts = w_f32[j].reshape(n_out, n_in)
                scale, zp = 0.0, 0
            else:
                q = (raw[j] >> np.uint64(24)) & np.uint64((1 << b) - 1)
                wts = q.astype(np.uint8 if b <= 8 else np.uint16).reshape(n_out, n_in)
                zp = 1 << (b - 1)
                scale = float(np.float32(2.0 * c / ((1 << b) - 1)))
            keep = None if keep_all is None else keep_all[j].reshape(n_out, n_in)
            models[j].layers.append(Layer(n_in, n_out, b, scale, zp, wts, keep, bias[j]))
    return models


def arch_draws(seed: int, ids: np.ndarray, n: int) -> np.ndarray:
    """n uniform (0,1) numbers per model id used for architecture choices."""
    return _unit24(stream_bits(stream_key(seed, np.asarray(ids, np.int64), 0, KIND_ARCH), n))


def draw_ids(seed: int, n: int, n_models: int, permutation: bool) -> np.ndarray:
    """Batch of image ids: a seeded permutation prefix, or draws with repeats."""
    r = stream_bits(stream_key(seed, 0, 0, KIND_IDS), max(n, n_models) if permutation else n)
    if permutation:
        order = np.argsort(r[:n_models], kind="stable").astype(np.int64)
        return order[:n].copy()
    return (r[:n] % np.uint64(n_models)).astype(np.int64)


@dataclass
class Workload:
    name: str
    models: List[Model]
    image_ids: np.ndarray
    H: int
    W: int
    out_u8: bool
    w0: float = 30.0
    coord_lo: float = -1.0
    coord_hi: float = 1.0

    @property
    def n(self) -> int:
        return len(self.image_ids)


def _uniform_models(seed, n_models, width, n_sine, hidden_bits, keep_prob, code_all=False):
    ids = np.arange(n_models)
    n_lin = n_sine + 1
    layer_bits = []
    a = arch_draws(seed, ids, n_lin)
    for l in range(n_lin):
        inner = 0 < l < n_lin - 1
        if hidden_bits is None or not (inner or code_all):
            layer_bits.append(0)
        elif isinstance(hidden_bits, int):
            layer_bits.append(hidden_bits)
        else:
            hb = np.asarray(hidden_bits)
            layer_bits.append(hb[np.minimum((a[:, l] * len(hb)).astype(int), len(hb) - 1)])
    out: List[Model] = []
    step = 2048
    for s in range(0, n_models, step):
        sl = slice(s, min(n_models, s + step))
        lb = [b if np.isscalar(b) else b[sl] for b in layer_bits]
        out.extend(make_models(seed, ids[sl], width, n_sine, lb, keep_prob))
    return out


RAGGED_WIDTHS = (24, 32, 40, 48, 64)
RAGGED_DEPTHS = (3, 4, 5, 6)


def ragged_pool(seed: int, n_models: int) -> List[Model]:
    """Pool of the ragged workload: width, depth, sparsity and per-layer bits per model."""
    ids = np.arange(n_models)
    a = arch_draws(seed, ids, 16)
    wi = np.minimum((a[:, 0] * len(RAGGED_WIDTHS)).astype(int), len(RAGGED_WIDTHS) - 1)
    di = np.minimum((a[:, 1] * len(RAGGED_DEPTHS)).astype(int), len(RAGGED_DEPTHS) - 1)
    sparsity = 0.3 + 0.5 * a[:, 2]
    bits = np.where(a[:, 3:3 + 8] < 0.5, 6, 8)
    models: List[Optional[Model]] = [None] * n_models
    for w_i, w in enumerate(RAGGED_WIDTHS):
        for d_i, d in enumerate(RAGGED_DEPTHS):
            sel = np.nonzero((wi == w_i) & (di == d_i))[0]
            for s in range(0, len(sel), 2048):
                part = sel[s:s + 2048]
                lb = [0] + [bits[part, l] for l in range(1, d)] + [0]
                ms = make_models(seed, part, w, d, lb, 1.0 - sparsity[part])
                for i, m in zip(part, ms):
                    models[i] = m
    return models  # type: ignore[return-value]


def workload(k: int, n_images: Optional[int] = None, pool: Optional[int] = None,
             H: Optional[int] = None, W: Optional[int] = None) -> Workload:
    """The five benchmark workloads (k = 1..5); seed = k - 1.

    `n_images`, `pool`, `H`, `W` shrink a workload for tests without changing
    the per-model recipe (model i of a shrunk pool equals model i of the full one).
    """
    seed = k - 1
    if k == 1:
        n = n_images or 64
        ms = _uniform_models(seed, n, 20, 3, None, None)
        return Workload("cfg1 64x32x32 2-20x3-3 fp32 dense", ms, draw_ids(seed, n, n, True), H or 32, W or 32, False)
    if k == 2:
        n = n_images or 4096
        ms = _uniform_models(seed, n, 32, 4, 8, 0.5)
        return Workload("cfg2 4096x32x32 2-32x4-3 q8 p50", ms, draw_ids(seed, n, n, True), H or 32, W or 32, False)
    if k == 3:
        n = n_images or 1024
        ms = _uniform_models(seed, n, 48, 5, (6, 8), 0.4)
        return Workload("cfg3 1024x64x64 2-48x5-3 q6/8 p60", ms, draw_ids(seed, n, n, True), H or 64, W or 64, False)
    if k == 4:
        n = n_images or 256
        ms = _uniform_models(seed, n, 64, 6, 8, 0.3)
        return Workload("cfg4 256x224x224 2-64x6-3 q8 p70", ms, draw_ids(seed, n, n, True), H or 224, W or 224, True)
    if k == 5:
        n = n_images or 1024
        p = pool or 50000
        ms = ragged_pool(seed, p)
        return Workload("cfg5 1024x128x128 ragged pool", ms, draw_ids(seed, n, p, False), H or 128, W or 128, False)
    raise ValueError("workload k must be 1..5")


def dense_flop_per_pixel(m: Model) -> int:
    """2 * sum(in*out) over the linear layers with their true widths."""
    return 2 * sum(l.n_in * l.n_out for l in m.layers)


# ---- inputs of the encode side: target images and initial weights ---------------------------

KIND_IMAGE = 4
KIND_INIT = 5


def images(seed: int, n: int, H: int, W: int) -> np.ndarray:
    """n procedural RGB images [n, 3, H, W] float32 in [0, 1]: a few smooth waves, a ramp and a soft-edged
    disc per channel (object boundaries are what INRs find hard).  Stand-ins for the paper's photographs:
    same shapes and value range, no dataset item reproduced."""
    ys = (np.arange(H, dtype=np.float64) + 0.5) / H
    xs = (np.arange(W, dtype=np.float64) + 0.5) / W
    Y, X = np.meshgrid(ys, xs, indexing="ij")
    out = np.empty((n, 3, H, W), dtype=np.float32)
    u = _unit24(stream_bits(stream_key(seed, np.arange(n), 0, KIND_IMAGE), 3 * 16)).reshape(n, 3, 16)
    for i in range(n):
        for c in range(3):
            r = u[i, c]
            img = 0.5 + 0.25 * (r[0] - 0.5) + 0.3 * (r[1] - 0.5) * (X - 0.5) + 0.3 * (r[2] - 0.5) * (Y - 0.5)
            for k in range(3):
                fx, fy, ph, am = 1 + 5 * r[3 + 4 * k], 1 + 5 * r[4 + 4 * k], 2 * math.pi * r[5 + 4 * k], 0.08 + 0.1 * r[6 + 4 * k]
                img = img + am * np.sin(2 * math.pi * (fx * X + fy * Y) + ph)
            cx, cy, rad = 0.2 + 0.6 * r[15], 0.2 + 0.6 * r[14], 0.1 + 0.2 * r[13]
            d = np.sqrt((X - cx) ** 2 + (Y - cy) ** 2)
            img = img + 0.25 * (r[12] - 0.5) * 2 / (1 + np.exp((d - rad) * 40.0))
            out[i, c] = np.clip(img, 0.0, 1.0)
    return out


def init_params(seed: int, widths: Sequence[int], n: int, w0: float = 30.0) -> np.ndarray:
    """Initial parameter vectors [n, n_params] float32 in the layout of the fit API (per layer W then b):
    first layer U(-1/d_in, 1/d_in), other weights U(+-sqrt(6/d_in)/w0), biases U(+-1/sqrt(d_in))/w0."""
    parts = []
    for l in range(len(widths) - 1):
        nin, nout = widths[l], widths[l + 1]
        bw = 1.0 / nin if l == 0 else math.sqrt(6.0 / nin) / w0
        bb = 1.0 / math.sqrt(nin) / w0
        uw = _unit24(stream_bits(stream_key(seed, np.arange(n), l, KIND_INIT), nout * nin))
        ub = _unit24(stream_bits(stream_key(seed, np.arange(n), l + 64, KIND_INIT), nout))
        parts.append((2 * uw - 1) * bw)
        parts.append((2 * ub - 1) * bb)
    return np.concatenate(parts, axis=1).astype(np.float32)


# ---- decode workloads with the paper's own model shapes (Sec. VI-A) -----------------------------

PAPER_SHAPES = {
    # name: (sine layers, width, image side, batch size of the backbone run, fraction of weights kept)
    "cifar": (2, 15, 32, 128, 1.0 - 0.156),       # "3 layers with 15 hidden dimensions", 32x32, 15.6 % pruned on average
    "flowers": (9, 32, 224, 64, 1.0 - 0.242),     # "10 layers with 32 hidden dimensions", 24.2 % pruned
    "imagenet": (9, 40, 224, 64, 1.0 - 0.255),    # "10 layers with 40 hidden dimensions", 25.5 % pruned
}


def paper_workload(name: str, n_images: Optional[int] = None, pool: int = 1024) -> Workload:
    """A batch drawn from a pool of models of one of the paper's three shapes: 8-bit hidden layers, first and
    last layer fp32 (Sec. IV-B), the average pruning ratio the paper reports (Sec. IV-A), coordinates on 0..1
    (Sec. III-A).  Batch size defaults to the one of the paper's backbone runs (Sec. VI-A)."""
    n_sine, width, side, batch, keep = PAPER_SHAPES[name]
    n = n_images or batch
    ms = _uniform_models(100 + len(name), pool, width, n_sine, 8, keep)
    ids = draw_ids(100 + len(name), n, pool, False)
    return Workload(f"paper {name}: {n}x{side}x{side} 2-{width}x{n_sine}-3 q8 keep {keep:.3f}", ms, ids, side, side, False,
                    30.0, 0.0, 1.0)
