"""Writes tests/golden/oracle_tiny_case.json: the oracle's own results on one tiny seeded input.

The file pins the oracle's arithmetic against accidental change (a later edit of oracle/vp_oracle.py
that alters a value must also regenerate this file, visibly).  It is written by this script, which
calls only the oracle and the seeded input generators; nothing in it comes from the GPU path, and
the paper prints no values for these layers that could be stored instead.

Usage:  python tests/golden/make_oracle_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import synth_inputs as si  # noqa: E402
from oracle import vp_oracle as oc  # noqa: E402

CASE = dict(N=6, h=5, V=12, p=3, seed=20241105)


def compute():
    H, Ws, labels = si.small_output_case(CASE["N"], CASE["h"], CASE["V"], CASE["p"], "f32", seed=CASE["seed"], w_std=0.5)
    X, W = si.as_f64(H), [si.as_f64(w) for w in Ws]
    a1 = oc.output_layer_alg1(X, W, labels)
    a2 = oc.output_layer_alg2(X, W, labels)
    ids = si.uniform_ids(CASE["N"], CASE["V"], CASE["seed"], stream=si.STREAM_PERM)
    g = si.as_f64(si.normal((CASE["N"], CASE["h"]), 1.0, "f32", CASE["seed"], si.STREAM_GRAD))
    dE = oc.embed_bwd(g, ids, 4, 4, np.zeros((4, CASE["h"])))
    return {"case": CASE, "labels": labels.tolist(), "ids": ids.tolist(), "loss": float(a1["loss"]),
            "m": a1["m"].tolist(), "sum": a1["sum"].tolist(), "m_loc": a1["m_loc"].tolist(),
            "sum_loc": a1["sum_loc"].tolist(), "dX": a1["dX"].tolist(), "dW_shard1": a1["dW"][1].tolist(),
            "alg2_dX": a2["dX"].tolist(), "alg2_A0": a2["A"][0].tolist(), "embed_bwd_shard1": dE.tolist()}


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_tiny_case.json")
    with open(out, "w") as f:
        json.dump(compute(), f, indent=1)
    print("wrote", out)
