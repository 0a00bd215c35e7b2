#!/usr/bin/env python3
"""Writes the stored expected values of the full-size parity tests.

Calls only the CPU oracle (oracle/) and the seeded input generators; nothing from the
HIP package is imported.  For each config it runs ONE HPP-Round (all M micro-batches in
1F1B order, then the momentum-SGD update with a seeded non-zero initial velocity, so
the momentum term is exercised) and stores, as float32:
  y_idx/y      a seeded sample of stage-output entries (logits for a loss-tailed stage)
  loss         the mini-batch mean loss (loss-tailed stages)
  dx_idx/dx    a seeded sample of input-gradient entries (flat indices into [M*B, ...])
  per parameter tensor: its L2 norm and a seeded sample of entries of the accumulated
  gradient G (before the update) and of the updated weights W.
Usage:  python tests/golden/make_golden.py cfg2 [cfg3 ...]
"""
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from asteroid_workloads import gen, get_config  # noqa: E402
from oracle import OracleStage, run_round  # noqa: E402

MAX_PER_TENSOR = 1024
DX_SAMPLES = 1 << 16


def initial_velocity(cfg, n):
    """Seeded non-zero velocity, scaled so momentum*v is comparable to typical gradients."""
    rng = np.random.Generator(np.random.PCG64(cfg.seed + 7))
    return (rng.standard_normal(n) * 0.05).astype(np.float32)


def sample_indices(cfg, n, count, salt):
    rng = np.random.Generator(np.random.PCG64(cfg.seed * 1000 + salt))
    if n <= count:
        return np.arange(n, dtype=np.int64)
    return np.sort(rng.choice(n, size=count, replace=False)).astype(np.int64)


def make(name):
    cfg = get_config(name)
    inp = gen.make_inputs(cfg)
    st = OracleStage(cfg.layers, cfg.B, cfg.M, cfg.in_shape, cfg.layout, cfg.needs_input_grad,
                     storage="bf16" if cfg.dtype == "bf16" else "f64")
    st.set_params(inp["params"])
    v0 = initial_velocity(cfg, st.nparams)
    st.set_velocity(v0)
    target = inp["labels"] if cfg.loss_tail else inp["dy"]
    t0 = time.time()
    ys, loss, dxs = run_round(st, inp["x"], target, K=1)
    G = st.G.copy()
    st.step(cfg.lr, cfg.momentum)
    W = st.W
    y = np.concatenate(ys).ravel()
    yi = sample_indices(cfg, y.size, DX_SAMPLES, 2)
    out = {"y_idx": yi, "y": y[yi].astype(np.float32), "y_norm": np.float64(np.linalg.norm(y)),
           "loss": np.float64(loss if cfg.loss_tail else 0.0)}
    if cfg.needs_input_grad:
        dx = np.concatenate(dxs).ravel()
        idx = sample_indices(cfg, dx.size, DX_SAMPLES, 1)
        out["dx_idx"] = idx
        out["dx"] = dx[idx].astype(np.float32)
        out["dx_norm"] = np.float64(np.linalg.norm(dx))
    off = 0
    for t, (li, pname, shape, _, _) in enumerate(gen.param_specs(cfg.layers)):
        n = int(np.prod(shape))
        idx = sample_indices(cfg, n, MAX_PER_TENSOR, 100 + t)
        key = "L%d.%s" % (li, pname)
        out["idx/" + key] = idx
        out["G/" + key] = G[off:off + n][idx].astype(np.float32)
        out["W/" + key] = W[off:off + n][idx].astype(np.float32)
        out["Gnorm/" + key] = np.float64(np.linalg.norm(G[off:off + n]))
        off += n
    out["G_rms"] = np.float64(np.sqrt(np.mean(G * G)))
    path = os.path.join(HERE, "%s_full.npz" % name)
    np.savez_compressed(path, **out)
    print("%s: %d params, oracle round %.1f s -> %s (%.1f KB)" %
          (name, st.nparams, time.time() - t0, path, os.path.getsize(path) / 1024), flush=True)


if __name__ == "__main__":
    for n in sys.argv[1:]:
        make(n)
