"""Pins of the encode-side oracle (oracle/fit_oracle.c) against things other than itself:
finite differences, the decode oracle, closed forms, the paper's printed schedule pieces."""
import json
import os
import types

import numpy as np
import pytest

from oracle import fit_oracle as fo
from oracle import oracle as dec

HERE = os.path.dirname(os.path.abspath(__file__))


def rand_params(widths, rng, scale=1.0):
    ps = []
    for l in range(len(widths) - 1):
        nin, nout = widths[l], widths[l + 1]
        bound = 0.5 if l == 0 else np.sqrt(6.0 / nin) / 30.0
        ps.append(rng.uniform(-bound, bound, nout * nin) * scale)
        ps.append(rng.uniform(-0.1, 0.1, nout))
    return np.concatenate(ps)


def as_model(widths, params, keep=None):
    """The same network as a decode-oracle model (raw fp32 layers)."""
    layers, off = [], 0
    for l in range(len(widths) - 1):
        nin, nout = widths[l], widths[l + 1]
        w = params[off:off + nout * nin].reshape(nout, nin).astype(np.float32)
        k = None if keep is None else keep[off:off + nout * nin].reshape(nout, nin).astype(np.uint8)
        off += nout * nin
        b = params[off:off + nout].astype(np.float32)
        off += nout
        layers.append(types.SimpleNamespace(n_in=nin, n_out=nout, bits=0, scale=1.0, zp=0, weights=w, keep=k, bias=b))
    return types.SimpleNamespace(layers=layers)


def test_forward_equals_decode_oracle():
    rng = np.random.default_rng(0)
    widths = [2, 7, 5, 6, 3]
    p = rand_params(widths, rng).astype(np.float32).astype(np.float64)     # fp32-representable
    keep = (rng.uniform(size=p.size) < 0.7).astype(np.uint8)
    for lo, hi in ((-1.0, 1.0), (0.0, 1.0)):
        for kp in (None, keep):
            kd = None
            if kp is not None:                # the decode model prunes weights only; keep the biases
                kd = kp.copy()
                off = 0
                for l in range(len(widths) - 1):
                    off += widths[l] * widths[l + 1]
                    kd[off:off + widths[l + 1]] = 1
                    off += widths[l + 1]
            got = fo.forward(widths, p, 5, 9, keep=kd, lo=lo, hi=hi)
            want = dec.decode([as_model(widths, p, kd)], np.array([0]), 5, 9, lo=lo, hi=hi, clamp=False)[0]
            np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_loss_of_zero_weights_is_bias_error():
    widths = [2, 4, 3]
    p = np.zeros(fo.n_params(widths))
    p[-3:] = [0.1, 0.5, -0.2]
    tgt = np.random.default_rng(1).uniform(0, 1, (3, 3, 4))
    loss, _ = fo.loss_grad(widths, p, tgt, loss_scale=1.0)
    want = sum(((p[-3 + k] - tgt[k]) ** 2).sum() for k in range(3))
    assert abs(loss - want) < 1e-12
    loss_mean, _ = fo.loss_grad(widths, p, tgt)
    assert abs(loss_mean - want / tgt.size) < 1e-14


@pytest.mark.parametrize("masked", [False, True])
def test_gradient_matches_central_differences(masked):
    rng = np.random.default_rng(2)
    widths = [2, 5, 4, 3]
    p = rand_params(widths, rng, scale=3.0)
    tgt = rng.uniform(0, 1, (3, 4, 5))
    keep = (rng.uniform(size=p.size) < 0.6).astype(np.uint8) if masked else None
    loss, g = fo.loss_grad(widths, p, tgt, keep)
    pe = p if keep is None else p * keep
    for i in range(p.size):
        if keep is not None and not keep[i]:
            assert g[i] == 0.0
            continue
        h = 1e-6
        a, b = pe.copy(), pe.copy()
        a[i] += h
        b[i] -= h
        fd = (fo.loss_grad(widths, a, tgt, keep, want_grad=False)[0] - fo.loss_grad(widths, b, tgt, keep, want_grad=False)[0]) / (2 * h)
        assert abs(fd - g[i]) <= 1e-7 * max(1.0, abs(g[i])) + 2e-9, (i, fd, g[i])


def test_output_bias_gradient_closed_form():
    rng = np.random.default_rng(3)
    widths = [2, 6, 3]
    p = rand_params(widths, rng)
    tgt = rng.uniform(0, 1, (3, 6, 4))
    _, g = fo.loss_grad(widths, p, tgt, loss_scale=1.0)
    f = fo.forward(widths, p, 6, 4)
    np.testing.assert_allclose(g[-3:], 2.0 * (f - tgt).sum(axis=(1, 2)), rtol=1e-12)


def test_adam_first_steps_closed_form():
    rng = np.random.default_rng(4)
    g = rng.normal(size=50)
    p0 = rng.normal(size=50)
    p, m, v = p0.copy(), np.zeros(50), np.zeros(50)
    fo.adam_step(p, m, v, g, 1, 1e-3, eps=1e-8)
    np.testing.assert_allclose(p, p0 - 1e-3 * g / (np.abs(g) + 1e-8), rtol=1e-13)
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-13)
    np.testing.assert_allclose(v, 0.001 * g * g, rtol=1e-12)
    p1 = p.copy()
    fo.adam_step(p, m, v, g, 2, 1e-3, eps=1e-8)          # same gradient again: bias-corrected moments are still g, g^2
    np.testing.assert_allclose(p, p1 - 1e-3 * g / (np.abs(g) + 1e-8), rtol=1e-12)
    keep = np.ones(50, dtype=np.uint8)
    keep[::3] = 0
    p, m, v = p0.copy(), np.zeros(50), np.zeros(50)
    fo.adam_step(p, m, v, g, 1, 1e-3, keep=keep)
    assert np.all(p[::3] == 0.0) and np.all(m[::3] == 0.0)


def test_cosine_schedule():
    assert fo.cosine_lr(5e-4, 0, 100) == 5e-4
    assert abs(fo.cosine_lr(5e-4, 50, 100) - 2.5e-4) < 1e-18
    assert abs(fo.cosine_lr(5e-4, 100, 100)) < 1e-18
    xs = [fo.cosine_lr(1.0, t, 64) for t in range(65)]
    assert all(a > b for a, b in zip(xs, xs[1:]))
    assert abs(fo.cosine_lr(1.0, 16, 64) - 0.5 * (1 + np.sqrt(0.5))) < 1e-15


def test_psnr_definition():
    a = np.zeros(1000)
    b = np.full(1000, 0.1)
    assert abs(fo.psnr(a, b) - 20.0) < 1e-12
    b = np.full(1000, 0.01)
    assert abs(fo.psnr(a, b) - 40.0) < 1e-12


def test_prune_ratio_matches_printed_pieces():
    cases = json.load(open(os.path.join(HERE, "golden", "prune_ratio.json")))["cases"]
    for sched, psnr, want in cases:
        assert abs(fo.prune_ratio(sched, psnr) - want) < 1e-12, (sched, psnr)
    for sched, brk in ((0, 30.0), (0, 35.0), (1, 35.0), (1, 40.0), (2, 35.0), (2, 40.0)):      # continuous at the breaks
        assert abs(fo.prune_ratio(sched, brk - 1e-9) - fo.prune_ratio(sched, brk + 1e-9)) < 1e-9


def test_l1_mask_definition():
    rng = np.random.default_rng(5)
    w = rng.normal(size=200)
    for ratio in (0.0, 0.2, 0.255, 0.4, 1.0):
        keep = fo.l1_mask(w, ratio)
        n_pruned = int(round(ratio * 200))
        assert int((keep == 0).sum()) == n_pruned
        if 0 < n_pruned < 200:
            assert np.abs(w[keep == 0]).max() <= np.abs(w[keep == 1]).min()
        order = np.argsort(np.abs(w), kind="stable")
        want = np.ones(200, dtype=np.uint8)
        want[order[:n_pruned]] = 0
        assert np.array_equal(keep, want)
    ties = np.array([0.5, -0.5, 0.5, 0.1, -0.5])
    assert list(fo.l1_mask(ties, 0.6)) == [0, 0, 1, 0, 1]          # 3 pruned: the 0.1, then the first two of the tied
    # second round: ratio counts all entries, the first round's zeros go first and stay pruned
    k1 = fo.l1_mask(w, 0.2)
    k2 = fo.l1_mask(w * k1, 0.3, keep_in=k1)
    assert int((k2 == 0).sum()) == 60 and np.all(k2[k1 == 0] == 0)
    assert np.array_equal(k2, fo.l1_mask(w, 0.3))
    k3 = fo.l1_mask(w * k1, 0.1, keep_in=k1)                        # a smaller ratio cannot revive weights
    assert np.array_equal(k3, k1)


@pytest.mark.parametrize("bits", [2, 4, 6, 8])
def test_quantiser_properties(bits):
    rng = np.random.default_rng(6 + bits)
    w = rng.normal(scale=0.02, size=500)
    w[::50] = 0.0
    keep = (rng.uniform(size=500) < 0.7).astype(np.uint8)
    for kp in (None, keep):
        scale, zp, q = fo.quantize(w, bits, kp)
        qmax = 2 ** bits - 1
        sel = np.ones(500, bool) if kp is None else kp.astype(bool)
        assert scale == float(np.float32(scale)) and 0 <= zp <= qmax and q.max() <= qmax
        deq = scale * (q.astype(np.float64) - zp)
        assert np.abs(deq[sel] - w[sel]).max() <= 0.5 * scale * (1 + 1e-6) + 0.5 * scale      # zp rounding adds up to half a step
        assert np.all(q[sel & (w == 0.0)] == zp)                      # zero is exact
        if kp is not None:
            assert np.all(q[~sel] == zp)
        lo, hi = min(w[sel].min(), 0.0), max(w[sel].max(), 0.0)
        assert abs(scale - np.float32((hi - lo) / qmax)) == 0.0
        assert q[sel].min() <= 1 and q[sel].max() >= qmax - 1            # the range's end points reach the end codes
    scale, zp, q = fo.quantize(np.zeros(10), bits)
    assert scale == 1.0 and zp == 0 and np.all(q == 0)
    scale, zp, q = fo.quantize(np.full(10, 0.3), bits)                  # one-sided range still contains 0
    assert zp == 0 and np.all(q == 2 ** bits - 1)


def test_quantised_layer_decodes_like_the_decode_oracle():
    rng = np.random.default_rng(9)
    w = rng.normal(scale=0.03, size=(6, 5))
    scale, zp, q = fo.quantize(w, 8)
    layer = types.SimpleNamespace(n_in=5, n_out=6, bits=8, scale=np.float32(scale), zp=zp,
                                  weights=q.reshape(6, 5), keep=None, bias=np.zeros(6, np.float32))
    deq = dec.dequant(layer)
    np.testing.assert_allclose(deq, np.float32(scale) * (q.reshape(6, 5).astype(np.float64) - zp), rtol=1e-7)
    assert np.abs(deq - w).max() <= scale


def test_fit_reduces_loss_and_fits_a_constant():
    rng = np.random.default_rng(10)
    widths = [2, 8, 8, 3]
    ys, xs = np.mgrid[0:8, 0:8] / 8.0
    tgt = np.stack([0.5 + 0.4 * np.sin(3 * xs), 0.5 + 0.4 * np.cos(2 * ys), 0.3 + 0.5 * xs * ys])
    p0 = rand_params(widths, rng)
    p, losses = fo.fit(widths, p0, tgt, steps=300, lr0=5e-3)
    assert losses[-1] < 0.1 * losses[0]
    const = np.broadcast_to(np.array([0.2, 0.5, 0.9])[:, None, None], (3, 4, 4)).copy()
    p, losses = fo.fit([2, 4, 3], np.zeros(fo.n_params([2, 4, 3])), const, steps=400, lr0=2e-2)
    assert losses[-1] < 1e-6 and np.allclose(p[-3:], [0.2, 0.5, 0.9], atol=2e-3)


def _grad_matrix_form(widths, p, tgt, w0=30.0, lo=-1.0, hi=1.0):
    """The same loss gradient written with whole-image matrix products (second, independent statement)."""
    _, H, W = tgt.shape
    ys = lo + (hi - lo) * (2 * np.arange(H) + 1) / (2 * H)
    xs = lo + (hi - lo) * (2 * np.arange(W) + 1) / (2 * W)
    Y, X = np.meshgrid(ys, xs, indexing="ij")
    hs, zs, layers, off = [np.stack([X.ravel(), Y.ravel()])], [], [], 0
    for l in range(len(widths) - 1):
        nin, nout = widths[l], widths[l + 1]
        layers.append((p[off:off + nout * nin].reshape(nout, nin), p[off + nout * nin:off + nout * nin + nout]))
        off += nout * nin + nout
    for l, (w, b) in enumerate(layers):
        zs.append(w @ hs[-1] + b[:, None])
        if l < len(layers) - 1:
            hs.append(np.sin(w0 * zs[-1]))
    d = 2.0 / tgt.size * (zs[-1] - tgt.reshape(3, -1))
    gs = []
    for l in range(len(layers) - 1, -1, -1):
        gs.append((d @ hs[l].T, d.sum(axis=1)))
        if l > 0:
            d = (layers[l][0].T @ d) * w0 * np.cos(w0 * zs[l - 1])
    return np.concatenate([np.concatenate([gw.ravel(), gb]) for gw, gb in gs[::-1]])


def test_gradient_matches_matrix_form_on_deep_models():
    rng = np.random.default_rng(12)
    for widths, H, W in (([2] + [32] * 9 + [3], 12, 10), ([2, 24, 48, 32, 3], 7, 9)):
        p = rand_params(widths, rng)
        tgt = rng.uniform(0, 1, (3, H, W))
        _, g = fo.loss_grad(widths, p, tgt)
        want = _grad_matrix_form(widths, p, tgt)
        assert np.abs(g - want).max() <= 1e-11 * np.abs(want).max()
