"""Frozen values of a tiny decode (tests/golden/tiny_decode.json, written by the oracle alone).

The paper prints no worked decode example, so these are not the paper's numbers: they pin the
oracle against drift (CPU test) and give the GPU path a fixed target (GPU test)."""
import json
import os

import numpy as np
import pytest

from oracle import oracle
from paper_2306_16699_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))
GOLD = json.load(open(os.path.join(HERE, "golden", "tiny_decode.json")))


def unhex(xs, shape):
    return np.array([float.fromhex(v) for v in xs], dtype=np.float64).reshape(shape)


@pytest.mark.parametrize("case", GOLD["cases"], ids=lambda c: f"w{c['workload']}")
def test_oracle_reproduces_frozen_values(case):
    w = synth.workload(case["workload"], n_images=case["images"], pool=case["pool"], H=case["H"], W=case["W"])
    assert w.image_ids.tolist() == case["image_ids"]
    shape = (case["images"], 3, case["H"], case["W"])
    raw = oracle.decode(w.models, w.image_ids, case["H"], case["W"], clamp=False)
    # bit-for-bit up to libm's last place in sin: allow 4 ulp of the value scale
    assert np.abs(raw - unhex(case["raw"], shape)).max() <= 1e-15
    _, u8 = oracle.decode(w.models, w.image_ids, case["H"], case["W"], want_u8=True)
    assert u8.reshape(-1).tolist() == case["u8"]
    aff = np.tile(np.array(case["affine"]), (case["images"], 1))
    aug = oracle.decode(w.models, w.image_ids, case["H"], case["W"], affine=aff,
                        norm=(np.array(case["norm_scale"]), np.array(case["norm_shift"])))
    assert np.abs(aug - unhex(case["augmented"], shape)).max() <= 1e-14


@pytest.mark.gpu
@pytest.mark.parametrize("case", GOLD["cases"], ids=lambda c: f"w{c['workload']}")
def test_gpu_matches_frozen_values(case):
    import torch
    from paper_2306_16699_amd import rinr
    w = synth.workload(case["workload"], n_images=case["images"], pool=case["pool"], H=case["H"], W=case["W"])
    shape = (case["images"], 3, case["H"], case["W"])
    st = rinr.Store(rinr.pack(w.models))
    ids = torch.from_numpy(w.image_ids).cuda()
    aff = torch.tensor([case["affine"]] * case["images"], dtype=torch.float32, device="cuda")
    for mode in (0, rinr.FLAG_FP32_MFMA):
        raw = st.decode_batch_ex(ids, case["H"], case["W"], rinr.OUT_F32, mode | rinr.FLAG_NO_CLAMP).cpu().numpy()
        assert np.abs(raw - unhex(case["raw"], shape)).max() <= 1e-3
        u8 = st.decode_batch_ex(ids, case["H"], case["W"], rinr.OUT_U8, mode).cpu().numpy()
        assert np.abs(u8.reshape(-1).astype(int) - np.array(case["u8"])).max() <= 1
        aug = st.decode_batch_ex(ids, case["H"], case["W"], rinr.OUT_F32, mode, affine=aff,
                                 norm=(case["norm_scale"], case["norm_shift"])).cpu().numpy()
        assert np.abs(aug - unhex(case["augmented"], shape)).max() <= 4e-3     # 1e-3 x the largest norm scale
    st.close()
