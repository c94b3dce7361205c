#!/usr/bin/env python3
"""Writes tests/golden/c0_oracle_digest.json from the CPU oracle alone (it imports nothing
of the HIP path): for the tiny configuration c0 at 50% sparsity, per block the SHA-256 of the
selected index list, the selection margin, and a few sums and sampled values of the layer
output.  The paper prints no worked numeric example of Eq. 12-21 or of Alg. 1, so this file
is not an independent pin of the oracle (those are the closed forms, brute-force and library
cross-checks in test_oracle_pins.py); it makes any later change of the oracle's arithmetic
or of the input generator show up as a deliberate, reviewed change of this fixture.

    python tests/golden/make_c0_fixture.py
"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import ff_oracle as O                      # noqa: E402
from paper_2602_00397_amd import workloads as W        # noqa: E402

SAMPLES = [(0, 0), (1, 7), (63, 255), (64, 0), (130, 99), (255, 255), (200, 13), (17, 128)]


def digest():
    shp = W.CONFIGS["c0"]
    lt = W.make_layer(shp)
    x = W.bf16_to_f32(W.make_hidden(shp))
    f = {n: W.bf16_to_f32(getattr(lt, n)) for n in ("w_gate", "w_up", "w_down", "w1", "w2", "wc1", "wc2")}
    k = O.k_from_sparsity(shp.d_ffn, 0.5)
    ks = [k] * shp.n_blocks
    res = O.fastforward_layer(x, f["w_gate"], f["w_up"], f["w_down"].T, f["w1"], f["w2"], shp.block, ks,
                              wc1=f["wc1"].T, wc2=f["wc2"])
    return {
        "config": "c0", "k": int(k),
        "indices_sha256": [hashlib.sha256(np.asarray(i, dtype="<i4").tobytes()).hexdigest() for i in res.indices],
        "margins": [float(m) for m in res.margins],
        "y_sum": float(res.y.sum()), "y_l2": float(np.sqrt((res.y ** 2).sum())), "y_absmax": float(np.abs(res.y).max()),
        "y_samples": [[t, c, float(res.y[t, c])] for t, c in SAMPLES],
        "macs_ffn": int(res.macs_ffn), "macs_comp": int(res.macs_comp), "macs_predictor": int(res.macs_predictor),
    }


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c0_oracle_digest.json")
    with open(out, "w") as fh:
        json.dump(digest(), fh, indent=1)
        fh.write("\n")
    print("wrote", out)
