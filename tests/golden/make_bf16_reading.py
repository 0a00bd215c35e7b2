#!/usr/bin/env python3
"""Puts on record how far the reading "bf16 compute, fp32 accumulation" moves the result away from
the plain fp64 definition: the oracle in its two modes, storage="f64" (no rounding anywhere) and
storage="bf16" (weight operands and every layer output rounded to bf16, sums exact - the mode the
bf16 GPU kernels are scored against), on reduced-size stages of the two bf16 configurations, same
seeded inputs (already bf16-representable).  Writes tests/golden/bf16_reading.json:
  {case: {"y": .., "dx": .., "G_median": .., "G_max": ..}}   rel-L2 of the bf16-storage result, fp64 as reference.
Calls only oracle/ and the input generators.
Usage:  python tests/golden/make_bf16_reading.py
"""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import harness  # noqa: E402
from asteroid_workloads import configs as C  # noqa: E402
from asteroid_workloads import gen  # noqa: E402
from oracle import OracleStage, run_round  # noqa: E402

PATH = os.path.join(HERE, "bf16_reading.json")

CASES = {
    "cfg4_small": lambda: C.cfg4(B=3, M=2, hw=10, cin=128, c=256),
    "cfg4_tiny": lambda: C.cfg4(B=2, M=3, hw=12, cin=16, c=24),
    "cfg5_small": lambda: C.cfg5(B=2, M=2, S=64, d=128, heads=2, ffn=256, nlayers=2),
    "cfg5_one_layer": lambda: C.cfg5(B=1, M=3, S=32, d=512, heads=8, ffn=2048, nlayers=1),
}


def one(cfg, inp, storage):
    st = OracleStage(cfg.layers, cfg.B, cfg.M, cfg.in_shape, cfg.layout, cfg.needs_input_grad, storage=storage)
    st.set_params(inp["params"])
    ys, _, dxs = run_round(st, inp["x"], inp["dy"], K=1)
    return np.concatenate(ys).ravel(), np.concatenate(dxs).ravel(), st.G.copy()


def distance(name):
    cfg = CASES[name]()
    inp = gen.make_inputs(cfg, randomize_affine=True)
    y64, dx64, g64 = one(cfg, inp, "f64")
    y16, dx16, g16 = one(cfg, inp, "bf16")
    g_rms = float(np.sqrt(np.mean(g64 ** 2)))
    errs = [harness.grad_error(a, b, g_rms)[0] for (_, a), (_, b) in
            zip(harness.split_params(cfg.layers, g16), harness.split_params(cfg.layers, g64))]
    return {"y": harness.rel_l2(y16, y64), "dx": harness.rel_l2(dx16, dx64),
            "G_median": float(np.median(errs)), "G_max": float(max(errs))}


if __name__ == "__main__":
    data = {}
    for c in CASES:
        data[c] = distance(c)
        print(c, data[c], flush=True)
    json.dump(data, open(PATH, "w"), indent=1, sort_keys=True)
