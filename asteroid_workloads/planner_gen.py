"""Seeded synthetic profiler tables and device pools for the parallelism planner.

Shapes follow the paper's planning inputs (Sec. 3.3): L layers, N devices of a few speed
classes (its Jetson Nano / TX2 / NX pools differ by about 1 : 2 : 4 in speed and 4 : 8 : 8 GB in
memory), per-layer FP / BP time tables over batch sizes 0..B that are NOT proportional to the
batch size (small batches under-use a device), BP about twice FP, early layers with large
activations and small weights, late layers the reverse, and device-to-device bandwidths far
below memory speed.  All times are whole numbers (held in float64), so that sums taken in any
order agree exactly; sizes and bandwidths are whole numbers too.

Holds no planner arithmetic: it only draws the tables.
"""
import numpy as np


def planner_problem(seed, L, N, B, M, kind="affine", memory="loose", block=1):
    """Dict with tf, tb [N][L][B+1], a, act, w [L], u [N], bw [N][N], B, M, block.

    kind:   "linear"  t = c * beta                       (the assumption the paper argues against)
            "affine"  t = c * (beta + s_d)               (fixed under-utilisation cost per call)
            "stair"   t = c * g_d * ceil(beta / g_d)     (a device works in groups of g_d samples)
    memory: "loose"   every device could hold any stage at the full micro-batch
            "tight"   budgets near the footprint of a third of the model: caps bind
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    speed = rng.choice([1, 2, 4], size=N)
    cost = rng.integers(20, 200, size=L)                # work per sample of layer l
    over = rng.integers(1, 6, size=N)                   # affine: extra samples' worth per call
    group = rng.choice([1, 2, 4], size=N)               # stair: samples per hardware pass
    beta = np.arange(B + 1)
    tf = np.zeros((N, L, B + 1))
    tb = np.zeros((N, L, B + 1))
    for d in range(N):
        if kind == "linear":
            eff = beta.astype(np.int64)
        elif kind == "affine":
            eff = beta + over[d]
        elif kind == "stair":
            eff = group[d] * ((beta + group[d] - 1) // group[d])
        else:
            raise ValueError(kind)
        for l in range(L):
            unit = int(cost[l]) * (4 // int(speed[d]))
            tf[d, l] = unit * eff
            tb[d, l] = 2 * unit * eff + int(rng.integers(0, 8))
        tf[d, :, 0] = 0
        tb[d, :, 0] = 0
    depth = np.arange(L) / max(L - 1, 1)
    a = np.floor(4096 * (1.0 - 0.8 * depth) * rng.uniform(0.5, 1.5, size=L)).astype(np.int64) + 64
    act = a * rng.integers(1, 4, size=L)
    w = np.floor(1024 * (0.2 + 4.0 * depth) * rng.uniform(0.5, 1.5, size=L)).astype(np.int64) + 16
    full = 3 * w.sum() + (2 * N - 1) * B * act.sum()
    if memory == "loose":
        u = np.full(N, 2 * full, dtype=np.int64)
    elif memory == "tight":
        third = 3 * w.sum() + B * act.sum()
        u = (third * rng.uniform(0.25, 1.2, size=N)).astype(np.int64)
    else:
        raise ValueError(memory)
    bw = np.zeros((N, N))
    for d in range(N):
        for e in range(d + 1, N):
            bw[d, e] = bw[e, d] = float(1 << int(rng.integers(2, 7)))
    return dict(tf=tf, tb=tb, a=a.astype(np.float64), act=act.astype(np.float64),
                w=w.astype(np.float64), u=u.astype(np.float64), bw=bw, B=B, M=M, block=block)
