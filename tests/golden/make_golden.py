#!/usr/bin/env python3
"""Writes the stored expected values of the full-size parity tests.

Calls only the CPU oracle (oracle/) and the seeded input generators; nothing from the
HIP package is imported.  For each config it runs ONE HPP-Round (all M micro-batches in
1F1B order, then the momentum-SGD update with a seeded non-zero initial velocity, so
the momentum term is exercised) and stores, as float32:
  y_idx/y      a seeded sample of stage-output entries (logits for a loss-tailed stage)
  ys_idx/ys    a STRUCTURED set of stage-output entries: the places a kernel's tiling can get
               wrong without an unbiased sample noticing (see structured_indices)
  loss         the mini-batch mean loss (loss-tailed stages)
  dx_idx/dx, dxs_idx/dxs   the same two sets for the input gradient (flat indices into [M*B, ...])
  per parameter tensor: its L2 norm and entries of the accumulated gradient G (before the
  update) and of the updated weights W - the whole tensor up to 4096 entries, else its first and
  last 64 entries and a seeded sample.
For the bf16 configs (oracle mode storage="bf16": tensors rounded where the kernels round) a
second round with the plain fp64 oracle stores the same entries under f64/...: the tests print
the GPU's distance to the unrounded definition next to the scored one.
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
WHOLE_TENSOR = 4096
DX_SAMPLES = 1 << 16
GEMM_TILES = (128, 256, 392)   # row-tile heights and per-block row ranges of the matrix-core kernels


def initial_velocity(cfg, n):
    """Seeded non-zero velocity, scaled so momentum*v is comparable to typical gradients."""
    rng = np.random.Generator(np.random.PCG64(cfg.seed + 7))
    return (rng.standard_normal(n) * 0.05).astype(np.float32)


def sample_indices(cfg, n, count, salt):
    rng = np.random.Generator(np.random.PCG64(cfg.seed * 1000 + salt))
    if n <= count:
        return np.arange(n, dtype=np.int64)
    return np.sort(rng.choice(n, size=count, replace=False)).astype(np.int64)


def structured_indices(cfg, shape, layout, salt):
    """Deterministic flat indices into a tensor [M*B, *shape] (per-sample `shape`, memory order of
    `layout`), chosen where tilings break:
      every tensor: its first and last 512 entries;
      NHWC images / token matrices (rows = pixels or tokens of a micro-batch, the M dimension of the
        matrix products): for the first and the last micro-batch the first and last row, and the rows on
        either side of the first three and last three multiples of 128, 256 and 392 rows - all channels;
      NCHW images: for the first and last sample of the first and last micro-batch, of the first, the last
        and six seeded channels: the first and last row and the first and last column of the plane."""
    B, M = cfg.B, cfg.M
    per = int(np.prod(shape))
    total = M * B * per
    idx = [np.arange(min(512, total)), np.arange(max(0, total - 512), total)]
    if len(shape) == 1:
        pass
    elif layout in ("nhwc", "bsd"):
        if layout == "nhwc":
            c, h, w = shape        # logical (C, H, W); memory [H][W][C]
            rows_per_sample, row_len = h * w, c
        else:
            s, d = shape
            rows_per_sample, row_len = s, d
        rows_mb = B * rows_per_sample
        rows = {0, rows_mb - 1}
        for t in GEMM_TILES:
            ks = list(range(1, rows_mb // t + 1))
            for k in ks[:3] + ks[-3:]:
                for r in (k * t - 1, k * t):
                    if 0 <= r < rows_mb:
                        rows.add(r)
        rows = np.array(sorted(rows), dtype=np.int64)
        for mb in sorted({0, M - 1}):
            base = (mb * rows_mb + rows)[:, None] * row_len + np.arange(row_len)[None, :]
            idx.append(base.ravel())
    else:
        c, h, w = shape
        rng = np.random.Generator(np.random.PCG64(cfg.seed * 1000 + salt))
        chans = sorted({0, c - 1} | set(int(v) for v in rng.integers(0, c, size=6)))
        samples = sorted({0, B - 1, (M - 1) * B, M * B - 1})
        for n in samples:
            for ch in chans:
                base = (n * c + ch) * h * w
                idx.append(base + np.arange(w))                    # first row
                idx.append(base + (h - 1) * w + np.arange(w))      # last row
                idx.append(base + np.arange(h) * w)                # first column
                idx.append(base + np.arange(h) * w + (w - 1))      # last column
    return np.unique(np.concatenate(idx)).astype(np.int64)


def param_indices(cfg, n, t):
    if n <= WHOLE_TENSOR:
        return np.arange(n, dtype=np.int64)
    return np.unique(np.concatenate([np.arange(64), np.arange(n - 64, n),
                                     sample_indices(cfg, n, MAX_PER_TENSOR, 100 + t)])).astype(np.int64)


def one_round(cfg, inp, storage):
    st = OracleStage(cfg.layers, cfg.B, cfg.M, cfg.in_shape, cfg.layout, cfg.needs_input_grad, storage=storage)
    st.set_params(inp["params"])
    st.set_velocity(initial_velocity(cfg, st.nparams))
    target = inp["labels"] if cfg.loss_tail else inp["dy"]
    ys, loss, dxs = run_round(st, inp["x"], target, K=1)
    G = st.G.copy()
    st.step(cfg.lr, cfg.momentum)
    y = np.concatenate(ys).ravel()
    dx = np.concatenate(dxs).ravel() if cfg.needs_input_grad else None
    return y, loss, dx, G, st.W.copy(), st.nparams


def make(name):
    cfg = get_config(name)
    inp = gen.make_inputs(cfg)
    t0 = time.time()
    y, loss, dx, G, W, nparams = one_round(cfg, inp, "bf16" if cfg.dtype == "bf16" else "f64")
    f64 = one_round(cfg, inp, "f64") if cfg.dtype == "bf16" else None
    out_shape = gen.out_shape(cfg.layers, cfg.in_shape)
    yi = sample_indices(cfg, y.size, DX_SAMPLES, 2)
    ysi = structured_indices(cfg, out_shape, cfg.layout, 3)
    out = {"y_idx": yi, "y": y[yi].astype(np.float32), "ys_idx": ysi, "ys": y[ysi].astype(np.float32),
           "y_norm": np.float64(np.linalg.norm(y)), "loss": np.float64(loss if cfg.loss_tail else 0.0)}
    if f64:
        out["f64/y"] = f64[0][yi].astype(np.float32)
    if cfg.needs_input_grad:
        idx = sample_indices(cfg, dx.size, DX_SAMPLES, 1)
        dsi = structured_indices(cfg, cfg.in_shape, cfg.layout, 4)
        out["dx_idx"] = idx
        out["dx"] = dx[idx].astype(np.float32)
        out["dxs_idx"] = dsi
        out["dxs"] = dx[dsi].astype(np.float32)
        out["dx_norm"] = np.float64(np.linalg.norm(dx))
        if f64:
            out["f64/dx"] = f64[2][idx].astype(np.float32)
    off = 0
    for t, (li, pname, shape, _, _) in enumerate(gen.param_specs(cfg.layers)):
        n = int(np.prod(shape))
        idx = param_indices(cfg, n, t)
        key = "L%d.%s" % (li, pname)
        out["idx/" + key] = idx
        out["G/" + key] = G[off:off + n][idx].astype(np.float32)
        out["W/" + key] = W[off:off + n][idx].astype(np.float32)
        out["Gnorm/" + key] = np.float64(np.linalg.norm(G[off:off + n]))
        if f64:
            out["f64/G/" + key] = f64[3][off:off + n][idx].astype(np.float32)
        off += n
    out["G_rms"] = np.float64(np.sqrt(np.mean(G * G)))
    path = os.path.join(HERE, "%s_full.npz" % name)
    np.savez_compressed(path, **out)
    print("%s: %d params, oracle %.1f s -> %s (%.1f KB)" %
          (name, nparams, time.time() - t0, path, os.path.getsize(path) / 1024), flush=True)


if __name__ == "__main__":
    for n in sys.argv[1:]:
        make(n)
