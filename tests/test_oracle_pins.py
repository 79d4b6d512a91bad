"""Pins of the CPU oracle against things other than itself.

Each test fixes one part of the decode definition (Sec. III-A/B, IV-A, IV-B,
VI-A of the paper) by a closed form, exact arithmetic, an invariant, or brute
force, chosen so that a dropped term, a wrong sign or index, or a transposed
operand fails at least one of them.
"""
import math
from fractions import Fraction

import mpmath
import numpy as np
import pytest

from oracle import oracle, oracle_np
from paper_2306_16699_amd import synth
from paper_2306_16699_amd.synth import Layer, Model

W0 = 30.0


def raw_layer(w, b, keep=None):
    w = np.asarray(w, dtype=np.float32)
    return Layer(w.shape[1], w.shape[0], 0, 0.0, 0, w, keep, np.asarray(b, dtype=np.float32))


def px(k, n, lo=-1.0, hi=1.0):
    return lo + (hi - lo) * (2 * k + 1) / (2 * n)


# ---- dequantisation (Sec. IV-B): exact rational arithmetic, every code, bits 2..8 and 16
@pytest.mark.parametrize("bits", [2, 3, 4, 5, 6, 7, 8, 16])
def test_dequant_matches_exact_rational(bits):
    rng = np.random.default_rng(bits)
    nq = 1 << bits
    codes = np.arange(nq, dtype=np.uint16) if bits <= 8 else np.concatenate(
        [rng.integers(0, nq, 4096), [0, 1, nq // 2, nq - 1]]).astype(np.uint16)
    for zp in {0, 1, nq // 2, nq - 1}:
        for scale in [np.float32(1.0), np.float32(0.0123456789), np.float32(2.0 * math.sqrt(6 / 64) / 30 / (nq - 1)),
                      np.float32(rng.uniform(1e-6, 3.0))]:
            ly = Layer(len(codes), 1, bits, float(scale), zp, codes.reshape(1, -1), None, np.zeros(1, np.float32))
            got = oracle.dequant(ly).reshape(-1)
            sc = Fraction(float(scale))
            for q, g in zip(codes.tolist(), got.tolist()):
                exact = sc * (q - zp)
                want = float(np.float32(float(exact)))     # exact fits a double; one rounding to fp32
                assert g == want, (bits, zp, float(scale), q)
            assert got[list(codes).index(zp)] == 0.0 and not np.signbit(got[list(codes).index(zp)])
            assert np.array_equal(oracle_np.dequant(ly).reshape(-1), got)


def test_raw_fp32_layer_passes_through():
    w = np.array([[1.5, -2.25e-3], [3.0e5, 7.0e-9], [0.1, -0.3]], np.float32)
    got = oracle.dequant(raw_layer(w, [0, 0, 0]))
    assert np.array_equal(got, w.astype(np.float64))


# ---- pruning (Sec. IV-A): a pruned weight is exactly a zero weight
def test_pruned_equals_code_at_zero_point():
    w = synth.workload(3, n_images=3, H=7, W=5)
    a = oracle.decode(w.models, w.image_ids, w.H, w.W)
    models2 = []
    for m in w.models:
        ls = []
        for ly in m.layers:
            if ly.bits == 0:
                wt = np.where(ly.keep != 0, ly.weights, np.float32(0)).astype(np.float32)
            else:
                wt = np.where(ly.keep != 0, ly.weights, ly.zp).astype(ly.weights.dtype)
            ls.append(Layer(ly.n_in, ly.n_out, ly.bits, ly.scale, ly.zp, wt, None, ly.bias))
        models2.append(Model(ls))
    b = oracle.decode(models2, w.image_ids, w.H, w.W)
    assert np.array_equal(a, b)


def test_all_pruned_layer_gives_bias_preactivation():
    rng = np.random.default_rng(5)
    l0 = raw_layer(rng.uniform(-.5, .5, (4, 2)), rng.uniform(-.1, .1, 4))
    b1 = rng.uniform(-.1, .1, 4).astype(np.float32)
    l1 = raw_layer(rng.uniform(-.3, .3, (4, 4)), b1, keep=np.zeros((4, 4), np.uint8))
    wout = np.eye(3, 4, dtype=np.float32)
    l2 = raw_layer(wout, [0, 0, 0])
    out = oracle.decode([Model([l0, l1, l2])], [0], 3, 4, clamp=False)
    for c in range(3):
        assert np.allclose(out[0, c], math.sin(W0 * float(b1[c])), rtol=0, atol=1e-15)


# ---- one sine layer: closed form sum_j a_cj sin(w0 (b_jx x + b_jy y + c_j)) + d_c in multiprecision
def test_single_sine_layer_closed_form():
    rng = np.random.default_rng(11)
    wdt, H, Wd = 5, 4, 6
    B = rng.uniform(-.5, .5, (wdt, 2)).astype(np.float32)
    cb = rng.uniform(-.1, .1, wdt).astype(np.float32)
    A = rng.uniform(-.4, .4, (3, wdt)).astype(np.float32)
    d = rng.uniform(.2, .6, 3).astype(np.float32)
    out = oracle.decode([Model([raw_layer(B, cb), raw_layer(A, d)])], [0], H, Wd, clamp=False)
    mpmath.mp.dps = 40
    for i in range(H):
        for j in range(Wd):
            x = mpmath.mpf(2 * j + 1) / (2 * Wd) * 2 - 1
            y = mpmath.mpf(2 * i + 1) / (2 * H) * 2 - 1
            for c in range(3):
                v = mpmath.mpf(float(d[c]))
                for k in range(wdt):
                    v += mpmath.mpf(float(A[c, k])) * mpmath.sin(
                        30 * (mpmath.mpf(float(B[k, 0])) * x + mpmath.mpf(float(B[k, 1])) * y + mpmath.mpf(float(cb[k]))))
                assert abs(float(v) - out[0, c, i, j]) < 5e-14


# ---- all-zero weights: every pixel is clamp(output bias), exactly
def test_zero_weights_give_clamped_bias():
    bias = np.array([0.25, -0.5, 1.75], np.float32)
    m = Model([raw_layer(np.zeros((6, 2)), np.zeros(6)), raw_layer(np.zeros((6, 6)), np.zeros(6)),
               raw_layer(np.zeros((3, 6)), bias)])
    out, u8 = oracle.decode([m], [0, 0], 5, 3, want_u8=True)
    want = np.clip(bias.astype(np.float64), 0, 1)
    assert np.array_equal(out, np.broadcast_to(want[None, :, None, None], out.shape))
    assert np.array_equal(u8[0, :, 0, 0], np.array([64, 0, 255], np.uint8))   # 63.75 -> 64


# ---- zero first layer: spatially constant image with a hand-computable value
def test_zero_first_layer_constant_image():
    b0 = np.array([0.01, -0.02], np.float32)
    w1 = np.array([[0.3, -0.2]], np.float32)
    b1 = np.array([0.05], np.float32)
    wo = np.array([[0.5], [-0.25], [0.125]], np.float32)
    bo = np.array([0.4, 0.5, 0.6], np.float32)
    m = Model([raw_layer(np.zeros((2, 2)), b0), raw_layer(w1, b1), raw_layer(wo, bo)])
    out = oracle.decode([m], [0], 4, 4, clamp=False)
    h0 = [math.sin(W0 * float(b)) for b in b0]
    h1 = math.sin(W0 * (float(w1[0, 0]) * h0[0] + float(w1[0, 1]) * h0[1] + float(b1[0])))
    for c in range(3):
        assert np.allclose(out[0, c], float(wo[c, 0]) * h1 + float(bo[c]), rtol=0, atol=1e-15)


# ---- axis order and pixel-centre grid: channel 0 follows x (columns), channel 1 follows y (rows)
def test_axis_order_and_pixel_centres():
    g = np.float32((math.pi / 2) / W0)
    l0 = raw_layer([[g, 0], [0, g]], [0, 0])
    lo_ = raw_layer([[1, 0], [0, 1], [0, 0]], [0, 0, 0.5])
    H, Wd = 3, 8
    out = oracle.decode([Model([l0, lo_])], [0], H, Wd, clamp=False)
    for i in range(H):
        for j in range(Wd):
            assert abs(out[0, 0, i, j] - math.sin(W0 * float(g) * px(j, Wd))) < 1e-15
            assert abs(out[0, 1, i, j] - math.sin(W0 * float(g) * px(i, H))) < 1e-15
            assert out[0, 2, i, j] == 0.5
    assert np.allclose(out[0, 0], -out[0, 0][:, ::-1], atol=1e-15)      # x_j = -x_{W-1-j}
    assert np.allclose(out[0, 1], -out[0, 1][::-1, :], atol=1e-15)
    o2 = oracle.decode([Model([l0, lo_])], [0], 2, 2, clamp=False)       # W = 2: centres are exactly -1/2, +1/2
    assert abs(o2[0, 0, 0, 1] - math.sin(W0 * float(g) * 0.5)) < 1e-15
    assert abs(o2[0, 1, 1, 0] - math.sin(W0 * float(g) * 0.5)) < 1e-15
    # the paper's own coordinate range, 0..1 (Sec. III-A): centres are (2k+1)/(2n)
    o3 = oracle.decode([Model([l0, lo_])], [0], 2, 4, lo=0.0, hi=1.0, clamp=False)
    assert abs(o3[0, 0, 1, 2] - math.sin(W0 * float(g) * 0.625)) < 1e-15
    assert abs(o3[0, 1, 1, 2] - math.sin(W0 * float(g) * 0.75)) < 1e-15


# ---- resolution-free decode (Sec. III-B): a 3x finer pixel-centre grid contains the coarse one
def test_resolution_nesting():
    w = synth.workload(2, n_images=2, H=6, W=5)
    a = oracle.decode(w.models, w.image_ids, 6, 5, clamp=False)
    b = oracle.decode(w.models, w.image_ids, 18, 15, clamp=False)
    assert np.allclose(a, b[:, :, 1::3, 1::3], rtol=0, atol=1e-12)


# ---- 2x2 image, width 2, two sine layers: every expression written out by hand
def test_two_by_two_unrolled():
    A = np.array([[0.31, -0.17], [-0.05, 0.44]], np.float32)
    a = np.array([0.03, -0.07], np.float32)
    Bm = np.array([[0.012, -0.021], [0.033, 0.008]], np.float32)
    b = np.array([0.02, 0.09], np.float32)
    Cm = np.array([[0.5, -0.25], [0.125, 0.75], [-0.6, 0.3]], np.float32)
    c = np.array([0.45, 0.5, 0.55], np.float32)
    out = oracle.decode([Model([raw_layer(A, a), raw_layer(Bm, b), raw_layer(Cm, c)])], [0], 2, 2, clamp=False)
    f = float
    for i, y in ((0, -0.5), (1, 0.5)):
        for j, x in ((0, -0.5), (1, 0.5)):
            p0 = math.sin(30 * (f(A[0, 0]) * x + f(A[0, 1]) * y + f(a[0])))
            p1 = math.sin(30 * (f(A[1, 0]) * x + f(A[1, 1]) * y + f(a[1])))
            q0 = math.sin(30 * (f(Bm[0, 0]) * p0 + f(Bm[0, 1]) * p1 + f(b[0])))
            q1 = math.sin(30 * (f(Bm[1, 0]) * p0 + f(Bm[1, 1]) * p1 + f(b[1])))
            assert abs(out[0, 0, i, j] - (f(Cm[0, 0]) * q0 + f(Cm[0, 1]) * q1 + f(c[0]))) < 1e-15
            assert abs(out[0, 1, i, j] - (f(Cm[1, 0]) * q0 + f(Cm[1, 1]) * q1 + f(c[1]))) < 1e-15
            assert abs(out[0, 2, i, j] - (f(Cm[2, 0]) * q0 + f(Cm[2, 1]) * q1 + f(c[2]))) < 1e-15


# ---- sin periodicity: shifting a hidden bias by 2*pi/w0 changes nothing (w0 multiplies weight sum AND bias)
def test_bias_period():
    rng = np.random.default_rng(3)
    l0 = raw_layer(rng.uniform(-.5, .5, (3, 2)), rng.uniform(-.1, .1, 3))
    w1 = rng.uniform(-.3, .3, (3, 3)); b1 = rng.uniform(-.1, .1, 3)
    lo_ = raw_layer(rng.uniform(-.5, .5, (3, 3)), [0.5, 0.5, 0.5])
    a = oracle.decode([Model([l0, raw_layer(w1, b1), lo_])], [0], 5, 5, clamp=False)
    b1s = b1.astype(np.float32).astype(np.float64) + 2 * math.pi / W0
    m2 = Model([l0, raw_layer(w1, b1), lo_])
    m2.layers[1].bias = b1s           # keep as float64 so the shift is not rounded to fp32
    # the C oracle reads fp32 biases: use the numpy oracle for the shifted model
    b = oracle_np.decode([m2], [0], 5, 5, clamp=False)
    assert np.allclose(a, b, rtol=0, atol=1e-13)


# ---- deep, rectangular chains (2 -> 5 -> 7 -> 6 -> 4 -> 3): facts that hold whatever the weights are
def _deep_chain(rng, scale=1.0):
    widths = [2, 5, 7, 6, 4, 3]
    ws = [rng.uniform(-.4, .4, (widths[k + 1], widths[k])) * scale for k in range(5)]
    bs = [rng.uniform(-.1, .1, widths[k + 1]) * scale for k in range(5)]
    return ws, bs


def _model(ws, bs):
    return Model([raw_layer(w, b) for w, b in zip(ws, bs)])


@pytest.mark.parametrize("dec", [oracle.decode, oracle_np.decode])
def test_hidden_units_can_be_renumbered(dec):
    """Permuting the units of a hidden layer (its rows and bias, the next layer's columns) changes nothing:
    fails if a layer is read transposed or a bias is attached to the wrong unit, at any depth."""
    rng = np.random.default_rng(11)
    ws, bs = _deep_chain(rng)
    ref = dec([_model(ws, bs)], [0], 4, 3, clamp=False)
    for k in range(4):
        perm = rng.permutation(ws[k].shape[0])
        w2, b2 = [w.copy() for w in ws], [b.copy() for b in bs]
        w2[k], b2[k], w2[k + 1] = ws[k][perm], bs[k][perm], ws[k + 1][:, perm]
        assert np.allclose(dec([_model(w2, b2)], [0], 4, 3, clamp=False), ref, rtol=0, atol=1e-11), k     # the order of the sums changes: rounding, times w0 per layer


@pytest.mark.parametrize("dec", [oracle.decode, oracle_np.decode])
def test_sine_is_odd_in_every_hidden_layer(dec):
    """Negating a unit's incoming weights and bias and its outgoing weights changes nothing (sin(-t) = -sin t):
    fails if a hidden layer's activation is not an odd function (cosine, or a bias added after the sine)."""
    rng = np.random.default_rng(12)
    ws, bs = _deep_chain(rng)
    ref = dec([_model(ws, bs)], [0], 3, 5, clamp=False)
    for k in range(4):
        j = int(rng.integers(ws[k].shape[0]))
        w2, b2 = [w.copy() for w in ws], [b.copy() for b in bs]
        w2[k][j] *= -1; b2[k][j] *= -1; w2[k + 1][:, j] *= -1
        assert np.allclose(dec([_model(w2, b2)], [0], 3, 5, clamp=False), ref, rtol=0, atol=1e-14), k
    # the output layer is linear: negating an output row and its bias negates that channel
    w2, b2 = [w.copy() for w in ws], [b.copy() for b in bs]
    w2[4][1] *= -1; b2[4][1] *= -1
    out = dec([_model(w2, b2)], [0], 3, 5, clamp=False)
    assert np.allclose(out[:, 1], -ref[:, 1], rtol=0, atol=1e-14) and np.allclose(out[:, 0], ref[:, 0], rtol=0, atol=1e-14)


@pytest.mark.parametrize("dec", [oracle.decode, oracle_np.decode])
def test_small_signal_limit_is_the_matrix_chain(dec):
    """With arguments t = w0 z of size <= 2e-3 everywhere, sin t = t up to a relative t^2 / 6 <= 7e-7 per layer: the deep
    model is then the affine chain out = W4 w0 (W3 w0 (... w0 (W0 x + b0) ...) + b3) + b4, evaluated here with
    plain matrix algebra.  Fixes layer order, operand orientation and where w0 and the biases enter, at depth."""
    rng = np.random.default_rng(13)
    ws, bs = _deep_chain(rng, scale=1e-4)
    ws = [w.astype(np.float32).astype(np.float64) for w in ws]
    bs = [b.astype(np.float32).astype(np.float64) for b in bs]
    H, W = 3, 4
    out = dec([_model(ws, bs)], [0], H, W, clamp=False)
    for i in range(H):
        for j in range(W):
            h = np.array([px(j, W), px(i, H)])
            for k in range(4):
                h = W0 * (ws[k] @ h + bs[k])
                assert np.abs(h).max() < 2e-3
            want = ws[4] @ h + bs[4]
            assert np.allclose(out[0, :, i, j], want, rtol=0, atol=np.abs(want).max() * 1e-5 + 1e-12)
            assert np.abs(want - bs[4]).max() > 1e-9        # the chain's contribution is visible at this tolerance


# ---- uint8 conversion: nearest, monotone, exact at the ends
def test_uint8_rounding_properties():
    vals = np.array([0.0, 1.0, 0.5, 1 / 255, 0.5 / 255 + 1e-9, 0.5 / 255 - 1e-9, 2.5 / 255, 3.5 / 255, 0.999], np.float64)
    m_list = []
    for v in vals:
        m_list.append(Model([raw_layer(np.zeros((1, 2)), [0]), raw_layer(np.zeros((3, 1)), [v, v, v])]))
    for k, v in enumerate(vals):
        m_list[k].layers[1].bias = np.array([v, v, v], np.float32)
    out, u8 = oracle.decode(m_list, np.arange(len(vals)), 1, 1, want_u8=True)
    c = out[:, 0, 0, 0]
    assert np.all(np.abs(u8[:, 0, 0, 0].astype(np.float64) - 255 * c) <= 0.5)
    assert u8[0, 0, 0, 0] == 0 and u8[1, 0, 0, 0] == 255
    assert np.array_equal(u8[:, 0, 0, 0], oracle_np.to_u8(c))
    order = np.argsort(c)
    assert np.all(np.diff(u8[order, 0, 0, 0].astype(int)) >= 0)
    # ties go to even: 2.5 -> 2, 3.5 -> 4 when 255*c is exactly the tie
    t = Model([raw_layer(np.zeros((1, 2)), [0]), raw_layer(np.zeros((3, 1)), [0.5, 0.5, 0.5])])
    _, t8 = oracle.decode([t], [0], 1, 1, want_u8=True)
    assert t8[0, 0, 0, 0] == 128                     # 127.5 -> 128 (even)


# ---- clamp edges
def test_clamp_edges():
    m = Model([raw_layer(np.zeros((1, 2)), [0]), raw_layer(np.zeros((3, 1)), [-0.2, 0.3, 1.2])])
    a = oracle.decode([m], [0], 2, 2)
    assert np.all(a[0, 0] == 0.0) and np.all(a[0, 2] == 1.0) and np.all(a[0, 1] == float(np.float32(0.3)))
    b = oracle.decode([m], [0], 2, 2, clamp=False)
    assert np.all(b[0, 0] == float(np.float32(-0.2))) and np.all(b[0, 2] == float(np.float32(1.2)))


# ---- gather (Sec. III-B batch select): slot s shows model ids[s]; repeats give identical planes
def test_gather_with_repeats():
    w = synth.workload(5, n_images=6, pool=12, H=4, W=4)
    ids = np.array([7, 3, 7, 11, 0, 3])
    out = oracle.decode(w.models, ids, 4, 4)
    assert np.array_equal(out[0], out[2]) and np.array_equal(out[1], out[5])
    for s, i in enumerate(ids):
        assert np.array_equal(out[s], oracle.decode(w.models, [i], 4, 4)[0])
    with pytest.raises(ValueError):
        oracle.decode(w.models, [12], 4, 4)


# ---- two independent implementations agree on full-depth random models of every workload shape
@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_c_and_numpy_oracles_agree(k):
    w = synth.workload(k, n_images=4, pool=40, H=9, W=7)
    a, a8 = oracle.decode(w.models, w.image_ids, 9, 7, want_u8=True)
    b = oracle_np.decode(w.models, w.image_ids, 9, 7)
    assert np.abs(a - b).max() < 1e-12
    assert np.array_equal(a8, oracle_np.to_u8(a))
    an = oracle.decode(w.models, w.image_ids, 9, 7, clamp=False)
    bn = oracle_np.decode(w.models, w.image_ids, 9, 7, clamp=False)
    assert np.abs(an - bn).max() < 1e-12
    assert np.array_equal(np.clip(an, 0, 1), a)


def test_thread_count_does_not_change_result():
    w = synth.workload(2, n_images=9, H=8, W=8)
    assert np.array_equal(oracle.decode(w.models, w.image_ids, 8, 8, n_threads=1),
                          oracle.decode(w.models, w.image_ids, 8, 8, n_threads=4))


# ---- augmentation (Sec. III-B): affine map of the sampling grid + per-channel normalisation ---------------
def _aug_models():
    w = synth.workload(3, n_images=3, H=8, W=8)
    ms = []
    for m in w.models:      # spread the outputs over [0, 1] so the clamp and the normalisation both matter
        last = m.layers[-1]
        ms.append(Model(m.layers[:-1] + [Layer(last.n_in, last.n_out, 0, 0.0, 0, (last.weights * np.float32(120)).astype(np.float32),
                                               last.keep, (last.bias + np.float32(0.5)).astype(np.float32))]))
    return ms


def test_aug_identity_is_plain_decode():
    ms = _aug_models()
    ids = np.array([2, 0, 1, 0])
    ident = np.tile(np.array([1, 0, 0, 0, 1, 0], np.float64), (4, 1))
    a = oracle.decode(ms, ids, 6, 9)
    b = oracle.decode(ms, ids, 6, 9, affine=ident, norm=(np.ones(3), np.zeros(3)))
    assert np.array_equal(a, b)


def test_aug_flip_rotate_and_crop_against_plain_decode():
    ms = _aug_models()
    ids = np.array([0, 1, 2])
    n, S = 3, 8
    plain = oracle.decode(ms, ids, S, S, clamp=False)
    flip = np.tile(np.array([-1, 0, 0, 0, 1, 0], np.float64), (n, 1))          # x -> -x: mirrored columns
    assert np.allclose(oracle.decode(ms, ids, S, S, clamp=False, affine=flip), plain[:, :, :, ::-1], rtol=0, atol=1e-12)
    vflip = np.tile(np.array([1, 0, 0, 0, -1, 0], np.float64), (n, 1))         # y -> -y: mirrored rows
    assert np.allclose(oracle.decode(ms, ids, S, S, clamp=False, affine=vflip), plain[:, :, ::-1, :], rtol=0, atol=1e-12)
    rot = np.tile(np.array([0, -1, 0, 1, 0, 0], np.float64), (n, 1))           # (x', y') = (-y, x)
    got = oracle.decode(ms, ids, S, S, clamp=False, affine=rot)
    want = np.transpose(plain, (0, 1, 3, 2))[:, :, ::-1, :]                     # out[i][j] = plain[j][S-1-i]
    assert np.allclose(got, want, rtol=0, atol=1e-12)
    # crop + resize: the top-left quadrant at full resolution == that quadrant of a plain 2x decode
    crop = np.tile(np.array([0.5, 0, -0.5, 0, 0.5, -0.5], np.float64), (n, 1))
    big = oracle.decode(ms, ids, 2 * S, 2 * S, clamp=False)
    assert np.allclose(oracle.decode(ms, ids, S, S, clamp=False, affine=crop), big[:, :, :S, :S], rtol=0, atol=1e-12)
    # translation by one pixel pitch of the base grid shifts columns by one
    shift = np.tile(np.array([1, 0, 2.0 / S, 0, 1, 0], np.float64), (n, 1))
    assert np.allclose(oracle.decode(ms, ids, S, S, clamp=False, affine=shift)[:, :, :, :-1], plain[:, :, :, 1:], rtol=0, atol=1e-12)
    # per-slot maps are per slot: slot 1 flipped only
    mixed = np.tile(np.array([1, 0, 0, 0, 1, 0], np.float64), (n, 1)); mixed[1] = flip[1]
    got = oracle.decode(ms, ids, S, S, clamp=False, affine=mixed)
    assert np.array_equal(got[0], plain[0]) and np.array_equal(got[2], plain[2])
    assert np.allclose(got[1], plain[1][:, :, ::-1], rtol=0, atol=1e-12)


def test_aug_normalisation_is_per_channel_after_clamp():
    ms = _aug_models()
    ids = np.array([1, 2])
    plain = oracle.decode(ms, ids, 7, 5)                       # clamped
    assert (plain == 0).any() and (plain == 1).any()
    scale, shift = np.array([4.0, 0.5, -2.0]), np.array([-1.5, 0.25, 3.0])
    got = oracle.decode(ms, ids, 7, 5, norm=(scale, shift))
    want = plain * scale[None, :, None, None] + shift[None, :, None, None]
    assert np.allclose(got, want, rtol=0, atol=1e-15)
    raw = oracle.decode(ms, ids, 7, 5, clamp=False)
    got_raw = oracle.decode(ms, ids, 7, 5, clamp=False, norm=(scale, shift))
    assert np.allclose(got_raw, raw * scale[None, :, None, None] + shift[None, :, None, None], rtol=0, atol=1e-14)


def test_aug_c_and_numpy_oracles_agree():
    ms = _aug_models()
    rng = np.random.default_rng(8)
    ids = np.array([0, 2, 1, 1])
    aff = rng.uniform(-1.2, 1.2, (4, 6))
    nrm = (rng.uniform(0.5, 5, 3), rng.uniform(-2, 2, 3))
    a = oracle.decode(ms, ids, 6, 7, affine=aff, norm=nrm)
    b = oracle_np.decode(ms, ids, 6, 7, affine=aff, norm=nrm)
    assert np.abs(a - b).max() < 1e-12
