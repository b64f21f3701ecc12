"""Writes tests/golden/toy_oracle.json: the CPU oracle's results on the toy
workload (1 layer, d=256, r=64, E=16, top-2, T=512, fp32).

The paper prints no worked numeric example of its predictor, so this file is a
regression value for the oracle, not a paper value: it was produced after the
oracle passed every pin in tests/test_oracle_pins.py.  It calls only the oracle
and the input generator.

    python tests/golden/make_golden.py
"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2511_10676_amd import configs, datagen  # noqa: E402


def compute():
    w = configs.get("toy")
    lay = datagen.make_layer(w, 0, w.prefill_T[0])
    idx, probs, z = oracle.predict(lay.x, lay.W1, lay.W2, w.k)
    idx3, _, _ = oracle.predict(lay.x, lay.W1, lay.W2, w.k_over)
    counts, offsets, pos, active, n_active, n_invalid = oracle.group_by_expert(idx, w.E)
    return {
        "workload": "toy",
        "idx_sha256": hashlib.sha256(idx.tobytes()).hexdigest(),
        "ref_sha256": hashlib.sha256(lay.ref.tobytes()).hexdigest(),
        "idx_first_rows": idx[:8].tolist(),
        "logit_row0": [float(f"{v:.12e}") for v in z[0]],
        "probs_row0": [float(f"{v:.6e}") for v in probs[0]],
        "counts": counts.tolist(),
        "n_active": n_active,
        "score_k2_vs_ref": oracle.score(idx, lay.ref, w.E).tolist(),
        "score_k3_vs_ref": oracle.score(idx3, lay.ref, w.E).tolist(),
    }


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "toy_oracle.json")
    with open(out, "w") as f:
        json.dump(compute(), f, indent=1)
        f.write("\n")
    print("wrote", out)
