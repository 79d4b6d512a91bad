"""Writes tests/golden/tiny_decode.json: expected values of a tiny decode, computed by the CPU
oracle only (no GPU code is imported or run).  Run from the repository root:
    python tests/golden/make_golden.py
The inputs are seeded synthetic models (paper_2306_16699_amd.synth holds no decode arithmetic);
the paper prints no worked numerical example of a decode (Sec. III-B describes it in prose), so
this file freezes the oracle's own values: a test fails if the oracle's arithmetic ever drifts,
and the GPU tests compare against the frozen numbers as well."""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import oracle                      # noqa: E402
from paper_2306_16699_amd import synth         # noqa: E402

CASES = [  # (workload, images, H, W)
    (2, 2, 3, 4),
    (3, 2, 2, 5),
    (5, 3, 4, 3),
]


def build():
    out = {"note": "values from oracle/inr_oracle.c (fp64); regenerate with tests/golden/make_golden.py", "cases": []}
    for k, n, H, W in CASES:
        w = synth.workload(k, n_images=n, pool=8, H=H, W=W)
        raw = oracle.decode(w.models, w.image_ids, H, W, clamp=False)
        clamped, u8 = oracle.decode(w.models, w.image_ids, H, W, want_u8=True)
        aff = np.tile(np.array([0.8, -0.3, 0.1, 0.25, 0.9, -0.05]), (w.n, 1))
        aug = oracle.decode(w.models, w.image_ids, H, W, affine=aff, norm=(np.array([2.0, 3.0, 4.0]), np.array([-0.5, 0.0, 0.5])))
        out["cases"].append({"workload": k, "images": n, "pool": 8, "H": H, "W": W, "image_ids": w.image_ids.tolist(),
                             "raw": [float.hex(float(v)) for v in raw.reshape(-1)],
                             "u8": u8.reshape(-1).tolist(),
                             "affine": aff[0].tolist(), "norm_scale": [2.0, 3.0, 4.0], "norm_shift": [-0.5, 0.0, 0.5],
                             "augmented": [float.hex(float(v)) for v in aug.reshape(-1)]})
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_decode.json")
    with open(path, "w") as f:
        json.dump(build(), f, indent=0)
    print("wrote", path)
