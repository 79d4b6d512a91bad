"""Host-side checks of the C-ABI library: exports, pack/unpack round trip, validation.

No GPU call is made here.  Expected values come from the inputs themselves (round trip)
and from the CPU oracle's dequantisation.
"""
import ctypes as C
import re
import os

import numpy as np
import pytest

from oracle import oracle
from paper_2306_16699_amd import rinr, synth
from paper_2306_16699_amd.synth import Layer, Model

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "rinr.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(rinr_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(rinr.EXPORTS), declared ^ set(rinr.EXPORTS)
    L = rinr.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert b"rinr" in L.rinr_version()
    assert rinr.strerror(0) == "ok" and "NULL" in rinr.strerror(rinr.E_NULL)


def rand_model(rng, width, n_sine, bits_choices, keep_prob, code_all=False):
    dims = [2] + [width] * n_sine + [3]
    layers = []
    for l in range(len(dims) - 1):
        n_in, n_out = dims[l], dims[l + 1]
        inner = 0 < l < len(dims) - 2
        bits = int(rng.choice(bits_choices)) if (inner or code_all) else 0
        if bits == 0:
            w = rng.uniform(-0.5, 0.5, (n_out, n_in)).astype(np.float32)
            scale, zp = 0.0, 0
        else:
            w = rng.integers(0, 1 << bits, (n_out, n_in)).astype(np.uint8 if bits <= 8 else np.uint16)
            scale, zp = float(np.float32(rng.uniform(1e-4, 1e-2))), int(rng.integers(0, 1 << bits))
        keep = None if keep_prob is None else (rng.uniform(size=(n_out, n_in)) < keep_prob).astype(np.uint8)
        layers.append(Layer(n_in, n_out, bits, scale, zp, w, keep, rng.uniform(-.1, .1, n_out).astype(np.float32)))
    return Model(layers)


@pytest.mark.parametrize("seed", range(6))
def test_pack_unpack_round_trip_random(seed):
    rng = np.random.default_rng(seed)
    models = []
    for _ in range(12):
        kp = [None, 0.0, 0.3, 0.7, 1.0][int(rng.integers(0, 5))]
        models.append(rand_model(rng, int(rng.integers(1, 65)), int(rng.integers(1, 10)),
                                 [0, 2, 3, 4, 5, 6, 7, 8, 16], kp, code_all=bool(rng.integers(0, 2))))
    blob = rinr.pack(models)
    for mi, m in enumerate(models):
        for li, ly in enumerate(m.layers):
            u = rinr.unpack_layer(blob, mi, li)
            keep = np.ones((ly.n_out, ly.n_in), np.uint8) if ly.keep is None else ly.keep
            assert (u["n_in"], u["n_out"], u["bits"]) == (ly.n_in, ly.n_out, ly.bits)
            assert np.array_equal(u["keep"], keep)
            assert u["n_kept"] == int(keep.sum())
            assert np.array_equal(u["bias"], ly.bias)
            want = oracle.dequant(ly)                       # fp64 holding fp32 values
            assert np.array_equal(u["f32"].astype(np.float64), want)
            if ly.bits:
                assert u["zp"] == ly.zp and u["scale"] == np.float32(ly.scale)
                assert np.array_equal(u["codes"], np.where(keep != 0, ly.weights, 0))


def test_pack_unpack_exhaustive_tiny_shapes():
    """Every (in, out) in 1..9 for the one free-shaped layer, every bit width, a dense and a sparse mask."""
    rng = np.random.default_rng(99)
    for n_mid_in in range(1, 10):
        for n_mid_out in range(1, 10):
            for bits in (0, 2, 3, 5, 6, 8, 16):
                for kp in (None, 0.5):
                    dims = [2, n_mid_in, n_mid_out, 3]
                    layers = []
                    for l in range(3):
                        n_in, n_out = dims[l], dims[l + 1]
                        b = bits if l == 1 else 0
                        if b == 0:
                            w = rng.uniform(-1, 1, (n_out, n_in)).astype(np.float32)
                        else:
                            w = rng.integers(0, 1 << b, (n_out, n_in)).astype(np.uint8 if b <= 8 else np.uint16)
                        keep = None if kp is None else (rng.uniform(size=(n_out, n_in)) < kp).astype(np.uint8)
                        layers.append(Layer(n_in, n_out, b, 0.01 if b else 0.0, (1 << b) // 2 if b else 0, w, keep,
                                            rng.uniform(-1, 1, n_out).astype(np.float32)))
                    blob = rinr.pack([Model(layers)])
                    for li, ly in enumerate(layers):
                        u = rinr.unpack_layer(blob, 0, li)
                        assert np.array_equal(u["f32"].astype(np.float64), oracle.dequant(ly))
                        assert np.array_equal(u["bias"], ly.bias)


def test_pack_size_matches_format_arithmetic():
    w = synth.workload(4, n_images=3)
    blob = rinr.pack(w.models)
    n = len(w.models)
    expect = (64 + 16 * n + 15) // 16 * 16
    for m in w.models:
        rec = 32 * len(m.layers)
        for ly in m.layers:
            cnt = ly.n_in * ly.n_out
            kept = cnt if ly.keep is None else int(ly.keep.sum())
            cb = ly.bits or 32
            rec += (4 * ((cnt + 31) // 32) if ly.keep is not None else 0) + 4 * ((kept * cb + 31) // 32 + 1) + 4 * ly.n_out
        expect += (rec + 15) // 16 * 16
    assert blob.size == expect
    # storage is the point of the format (paper abstract): ~0.3 kept x 8 bit + 1 mask bit per hidden weight
    assert blob.size / n < 13000


def _one(layers):
    return [Model(layers)]


def _good():
    rng = np.random.default_rng(0)
    return rand_model(rng, 8, 2, [8], 0.5)


def test_pack_rejects_bad_models():
    def rc_of(models):
        with pytest.raises(rinr.RinrError) as e:
            rinr.pack(models)
        return e.value.code
    g = _good()
    m = Model(list(g.layers)); m.layers = m.layers[:1]
    assert rc_of([m]) == rinr.E_MODEL                                   # too few layers, last out != 3
    m = Model([Layer(3, 8, 0, 0, 0, np.zeros((8, 3), np.float32), None, np.zeros(8, np.float32))] + g.layers[1:])
    assert rc_of([m]) == rinr.E_MODEL                                   # first in != 2
    ly = g.layers[1]
    for bad_bits in (1, 9, 12, 32, -1):
        m = Model([g.layers[0], Layer(ly.n_in, ly.n_out, bad_bits, ly.scale, 0, ly.weights, ly.keep, ly.bias), g.layers[2]])
        assert rc_of([m]) == rinr.E_MODEL
    m = Model([g.layers[0], Layer(ly.n_in, ly.n_out, 8, ly.scale, 256, ly.weights, ly.keep, ly.bias), g.layers[2]])
    assert rc_of([m]) == rinr.E_MODEL                                   # zp out of range
    m = Model([g.layers[0], Layer(ly.n_in, ly.n_out, 6, ly.scale, 3, np.full((8, 8), 64, np.uint8), None, ly.bias), g.layers[2]])
    assert rc_of([m]) == rinr.E_MODEL                                   # code >= 2^bits
    m = Model([g.layers[0], Layer(ly.n_in, ly.n_out, 8, float("nan"), 3, ly.weights, ly.keep, ly.bias), g.layers[2]])
    assert rc_of([m]) == rinr.E_MODEL
    bb = ly.bias.copy(); bb[0] = np.inf
    m = Model([g.layers[0], Layer(ly.n_in, ly.n_out, 8, ly.scale, 3, ly.weights, ly.keep, bb), g.layers[2]])
    assert rc_of([m]) == rinr.E_MODEL
    wide = Layer(2, 65, 0, 0, 0, np.zeros((65, 2), np.float32), None, np.zeros(65, np.float32))
    m = Model([wide, Layer(65, 3, 0, 0, 0, np.zeros((3, 65), np.float32), None, np.zeros(3, np.float32))])
    assert rc_of([m]) == rinr.E_MODEL                                   # wider than RINR_MAX_WIDTH
    m = Model([g.layers[0], g.layers[2]])
    m.layers[1] = Layer(7, 3, 0, 0, 0, np.zeros((3, 7), np.float32), None, np.zeros(3, np.float32))
    assert rc_of([m]) == rinr.E_MODEL                                   # chain mismatch
    # a pruned out-of-range code or a pruned NaN weight is ignored, not an error
    keep = np.ones((8, 8), np.uint8); keep[0, 0] = 0
    codes = np.zeros((8, 8), np.uint8); codes[0, 0] = 255
    m = Model([g.layers[0], Layer(8, 8, 6, 0.01, 3, codes, keep, ly.bias), g.layers[2]])
    rinr.pack([m])
    with pytest.raises(rinr.RinrError) as e:
        rinr.pack([g], w0=float("inf"))
    assert e.value.code == rinr.E_ARG
    with pytest.raises(rinr.RinrError) as e:
        rinr.pack([g], coord_lo=1.0, coord_hi=1.0)
    assert e.value.code == rinr.E_ARG


def test_pack_null_and_small_buffer():
    L = rinr.lib()
    descs, hold = rinr.marshal_models([_good()])
    size = C.c_size_t(0)
    assert L.rinr_pack_size(descs, 1, None, None) == rinr.E_NULL
    assert L.rinr_pack_size(None, 1, None, C.byref(size)) == rinr.E_NULL
    assert L.rinr_pack_size(descs, -1, None, C.byref(size)) == rinr.E_ARG
    assert L.rinr_pack_size(descs, 1, None, C.byref(size)) == 0
    buf = np.zeros(size.value, np.uint8)
    assert L.rinr_pack(descs, 1, None, None, size.value) == rinr.E_NULL
    assert L.rinr_pack(descs, 1, None, buf.ctypes.data, size.value - 1) == rinr.E_SIZE
    assert L.rinr_pack(descs, 1, None, buf.ctypes.data, size.value) == 0
    # empty dataset packs to header only
    assert L.rinr_pack_size(None, 0, None, C.byref(size)) == 0 and size.value == 64


def test_unpack_rejects_corrupt_blobs():
    blob = rinr.pack([_good(), _good()])
    L = rinr.lib()

    def rc(b, model=0, layer=0):
        return L.rinr_unpack_layer(b.ctypes.data, b.size, model, layer, None, None, None, None, None, None)
    assert rc(blob) == 0
    assert rc(blob, 2, 0) == rinr.E_ARG and rc(blob, 0, 3) == rinr.E_ARG and rc(blob, -1, 0) == rinr.E_ARG
    b = blob.copy(); b[0] ^= 0xFF
    assert rc(b) == rinr.E_FORMAT                                        # magic
    b = blob.copy(); b[8] = 9
    assert rc(b) == rinr.E_FORMAT                                        # version
    assert rc(blob[:40].copy()) == rinr.E_FORMAT                         # truncated header
    assert rc(blob[:-16].copy()) == rinr.E_FORMAT                        # truncated body
    b = blob.copy(); b[64:72] = np.frombuffer(np.uint64(blob.size + 16).tobytes(), np.uint8)
    assert rc(b) == rinr.E_FORMAT                                        # record offset past the end
    b = blob.copy(); b[64 + 12] = 200
    assert rc(b) == rinr.E_FORMAT                                        # n_layers absurd
    off = int(np.frombuffer(blob[64:72].tobytes(), np.uint64)[0])
    b = blob.copy(); b[off + 32 + 16] ^= 1                               # n_kept of layer 1 no longer matches the mask
    assert rc(b) == rinr.E_FORMAT
    b = blob.copy(); b[off + 32 + 24: off + 32 + 28] = np.frombuffer(np.uint32(1 << 30).tobytes(), np.uint8)
    assert rc(b) == rinr.E_FORMAT                                        # code offset outside the record
