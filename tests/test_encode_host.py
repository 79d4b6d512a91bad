"""Host functions of the encode side (include/rinr_fit.h) against the encode oracle: bit-exact."""
import json
import os
import re

import numpy as np
import pytest

from oracle import fit_oracle as fo
from paper_2306_16699_amd import rinr, rinr_fit

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_fit_symbol():
    hdr = open(os.path.join(ROOT, "include", "rinr_fit.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(rinr_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(rinr_fit.EXPORTS), declared ^ set(rinr_fit.EXPORTS)
    L = rinr_fit.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_prune_ratio_matches_paper_pieces_and_oracle():
    cases = json.load(open(os.path.join(ROOT, "tests", "golden", "prune_ratio.json")))["cases"]
    for sched, psnr, want in cases:
        assert abs(rinr_fit.prune_ratio(sched, psnr) - want) < 1e-12
    for sched in (0, 1, 2):
        for psnr in np.linspace(0.0, 60.0, 601):
            assert rinr_fit.prune_ratio(sched, float(psnr)) == fo.prune_ratio(sched, float(psnr))
    assert np.isnan(rinr_fit.prune_ratio(3, 30.0)) and np.isnan(rinr_fit.prune_ratio(0, float("nan")))


def test_l1_mask_bit_exact():
    rng = np.random.default_rng(0)
    for n in (1, 7, 64, 1000):
        w = rng.normal(size=n).astype(np.float32)
        w[rng.integers(0, n, n // 5)] = 0.0
        if n > 10:
            w[5] = -w[3]                     # a tie in magnitude
        for ratio in (0.0, 0.2, 0.255, 0.4, 0.5, 1.0):
            k = rinr_fit.l1_mask(w, ratio)
            assert np.array_equal(k, fo.l1_mask(w.astype(np.float64), ratio)), (n, ratio)
            k2 = rinr_fit.l1_mask(w * k, min(1.0, ratio + 0.1), keep_in=k)
            assert np.array_equal(k2, fo.l1_mask((w * k).astype(np.float64), min(1.0, ratio + 0.1), keep_in=k))
    with pytest.raises(rinr.RinrError):
        rinr_fit.l1_mask(np.ones(4, np.float32), 1.5)
    with pytest.raises(rinr.RinrError):
        rinr_fit.l1_mask(np.ones(4, np.float32), float("nan"))
    assert rinr_fit.l1_mask(np.zeros(0, np.float32), 0.5).size == 0


@pytest.mark.parametrize("bits", [2, 3, 6, 8, 16])
def test_quantiser_bit_exact(bits):
    rng = np.random.default_rng(bits)
    for n, sc in ((1, 1.0), (33, 0.02), (4096, 0.01), (500, 3.0)):
        w = rng.normal(scale=sc, size=n).astype(np.float32)
        keep = (rng.uniform(size=n) < 0.7).astype(np.uint8)
        for kp in (None, keep):
            s, z, q = rinr_fit.quantize_layer(w, bits, kp)
            so, zo, qo = fo.quantize(w.astype(np.float64), bits, kp)
            assert float(s) == so and z == zo and np.array_equal(q, qo), (bits, n)
    s, z, q = rinr_fit.quantize_layer(np.zeros(5, np.float32), bits)
    assert float(s) == 1.0 and z == 0 and not q.any()
    with pytest.raises(rinr.RinrError):
        rinr_fit.quantize_layer(np.array([np.inf], np.float32), bits)
    with pytest.raises(rinr.RinrError):
        rinr_fit.quantize_layer(np.ones(3, np.float32), 9)
