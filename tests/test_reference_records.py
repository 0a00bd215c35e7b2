"""CPU checks of the two records the GPU parity bars lean on (both written by committed scripts
that call only the oracle, the input generators and PyTorch CPU):

  tests/golden/fp32_reference.json - what an independent fp32 implementation (PyTorch CPU fp32
    autograd) holds against the fp64 oracle on the deep BatchNorm stacks; the relaxed gradient bars
    of tests/test_parity_gpu.py are 1.5 x these figures (derived_bar);
  tests/golden/bf16_reading.json - how far the oracle's bf16-storage mode (the reading of "bf16
    compute, fp32 accumulation" the bf16 kernels are scored against) lies from the plain fp64
    definition.

The figures are recomputed here for the cases that take seconds and must agree with the stored ones.
"""
import importlib.util
import json
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _load(script):
    spec = importlib.util.spec_from_file_location(script, os.path.join(HERE, "golden", script + ".py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_fp32_reference_record_is_complete():
    ref = json.load(open(os.path.join(HERE, "golden", "fp32_reference.json")))
    for case in ("cfg3_small", "effnetb1_small", "resnet50_small", "cfg2_small", "cfg7_small",
                 "cfg2_full", "cfg7_full", "cfg3_full"):
        assert case in ref, case
        for k, v in ref[case].items():
            if k != "runs":
                assert np.isfinite(v) and v > 0, (case, k, v)
        assert len(ref[case]["runs"]) == 4
    # the point of the record: fp32 cannot hold the stated 1e-3 on the gradients of the deep stacks ...
    assert ref["cfg3_small"]["G_max"] > 1e-3 and ref["cfg3_full"]["G_median"] > 1e-3 and ref["cfg2_full"]["G_max"] > 1e-3
    # ... while shallow stages and every forward pass are far inside the stated tolerances
    assert ref["cfg2_small"]["G_max"] < 1e-4 and ref["cfg7_small"]["G_max"] < 1e-4
    assert all(ref[c]["y"] < 1e-4 for c in ref)


@pytest.mark.parametrize("case", ["cfg2_small", "cfg7_small", "cfg3_small"])
def test_fp32_reference_recomputed(case):
    mod = _load("make_fp32_reference")
    ref = json.load(open(mod.PATH))[case]
    got = mod.small_case(case)
    for k in ref:
        if k == "runs":
            continue
        # fp32 sums depend on the host's thread count and BLAS blocking: same magnitude, not same digits
        assert 0.4 * ref[k] <= got[k] <= 2.5 * ref[k], (case, k, got[k], ref[k])


def test_bf16_reading_record():
    mod = _load("make_bf16_reading")
    ref = json.load(open(mod.PATH))
    assert set(ref) == set(mod.CASES)
    for case in ("cfg4_tiny", "cfg5_small"):
        got = mod.distance(case)
        for k in ref[case]:
            assert got[k] == pytest.approx(ref[case][k], rel=1e-6), (case, k)
    # the size of the reading: ReLU masks and max-pool winners decided on bf16-rounded tensors move the
    # conv stage's gradients by several percent of their norm; the transformer stage (no such decisions)
    # stays within half a percent, the forward pass of both within one bf16 ulp of accumulated rounding
    assert 2e-2 < ref["cfg4_small"]["dx"] < 2e-1 and 2e-2 < ref["cfg4_small"]["G_max"] < 2e-1
    assert ref["cfg5_small"]["G_max"] < 1e-2 and ref["cfg5_small"]["dx"] < 1e-2
    assert all(ref[c]["y"] < 1e-2 for c in ref)


def test_goldens_hold_structured_entries():
    for name in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "cfg6", "cfg7"):
        g = np.load(os.path.join(HERE, "golden", "%s_full.npz" % name))
        assert "ys_idx" in g and g["ys_idx"].size == g["ys"].size and g["ys_idx"].size >= 80
        assert g["ys_idx"][0] == 0                       # the very first entry ...
        if name not in ("cfg3",):                        # (cfg3: no input gradient)
            assert "dxs_idx" in g and g["dxs_idx"][0] == 0
        if name in ("cfg4", "cfg5"):                     # distance to the unrounded definition is on record
            assert "f64/y" in g and "f64/dx" in g and any(k.startswith("f64/G/") for k in g.files)
