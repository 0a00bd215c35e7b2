"""Profiler (Sec. 3.3 "DNN Model and Asteroid Profiler"): measures, with this library as the
executor, the tables the planner needs -- per layer l the output size a_l, the weight size w_l
and the FP / BP time t_f(beta), t_b(beta) over a set of batch sizes -- on the GPU it runs on.

A "layer" of the table is a profiling unit: the shortest run of consecutive layers that a
pipeline stage may start or end at (a convolution with its BatchNorm and activation, a whole
residual block, an attention or feed-forward block with its LayerNorm).  Sec. 5.7 "Planning
Overhead" suggests this granularity to keep the planner's search small.

Every time is measured by running the unit as a one-micro-batch stage through the C ABI
(asteroid_stage_forward / _backward) between HIP events on the stage's stream; nothing is
modelled.  Requires a GPU and the built library.

    python -m paper_2408_08015_amd.profiler --workload cfg3 --betas 1,2,4,8,16,32
"""
import argparse
import json
import sys

import numpy as np

from . import binding as A

_STARTS = ("conv2d", "res_begin", "se_begin", "mha", "global_avgpool")


def split_units(layers):
    """[(lo, hi)) runs of layer indices: cut in front of a convolution, a residual block, an
    attention layer, a squeeze-and-excitation block or the pooling of the classifier, never inside
    a residual or squeeze-and-excitation block."""
    cuts, depth = [0], 0
    for i, L in enumerate(layers):
        k = L["kind"]
        start = k in _STARTS or (k == "linear" and i > 0 and layers[i - 1]["kind"] != "global_avgpool")
        if i > 0 and depth == 0 and start:
            cuts.append(i)
        if k in ("res_begin", "se_begin"):
            depth += 1
        elif k in ("res_add", "se_scale"):
            depth -= 1
    cuts.append(len(layers))
    return [(cuts[i], cuts[i + 1]) for i in range(len(cuts) - 1)]


def _out_shape(layers, s):
    s = tuple(s)
    se, res = [], []
    for L in layers:
        k = L["kind"]
        if k == "se_begin":
            se.append(s)
        elif k == "se_scale":
            s = se.pop()
        elif k == "res_begin":
            res.append(s)
        elif k == "res_swap":
            s, res[-1] = res[-1], s
        elif k == "res_add":
            res.pop()
        elif k == "conv2d":
            c, h, w = s
            s = (L["cout"], (h + 2 * L["pad"] - L["k"]) // L["stride"] + 1,
                 (w + 2 * L["pad"] - L["k"]) // L["stride"] + 1)
        elif k == "maxpool2x2":
            s = (s[0], s[1] // 2, s[2] // 2)
        elif k == "maxpool3x3s2":
            s = (s[0], (s[1] - 1) // 2 + 1, (s[2] - 1) // 2 + 1)
        elif k == "global_avgpool":
            s = (s[0],)
        elif k == "linear":
            s = s[:-1] + (L["cout"],)
    return s


def _boundary(layout, per_sample, n):
    if layout == "nhwc" and len(per_sample) == 3:
        c, h, w = per_sample
        return (n, h, w, c)
    return (n,) + tuple(per_sample)


def time_unit(layers, in_shape, beta, dtype, layout, needs_input_grad, reps=20, warmup=3):
    """Median FP and BP time in ms of `layers` as a stage with one micro-batch of beta samples."""
    import torch
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    loss_tail = layers[-1]["kind"] == "softmax_ce"
    out = _out_shape(layers, in_shape)
    lay_out = layout if len(out) == len(in_shape) else "nchw"
    stream = torch.cuda.current_stream()
    st = A.Stage(layers, beta, 1, 1, in_shape, dtype, layout, needs_input_grad, stream=stream.cuda_stream)
    g = torch.Generator(device="cpu").manual_seed(1234)
    n = st.num_params
    if n:
        st.set_params((0.05 * torch.randn(n, generator=g)).numpy() + 0.5)
    x = torch.randn(_boundary(layout, in_shape, beta), generator=g).to(dev).to(tdt).contiguous()
    dx = torch.zeros_like(x) if needs_input_grad else None
    if loss_tail:
        labels = torch.randint(0, out[0], (beta,), generator=g, dtype=torch.int32).to(dev)
        y = torch.zeros((beta, out[0]), device=dev)
        dy, loss = None, torch.zeros(4, device=dev)
    else:
        labels, loss = None, None
        y = torch.zeros(_boundary(lay_out, out, beta), device=dev, dtype=tdt)
        dy = torch.randn(y.shape, generator=g).to(dev).to(tdt).contiguous()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(reps)]
    for r in range(-warmup, reps):
        if r >= 0:
            ev[r][0].record(stream)
        st.forward(0, x, labels, y, loss)
        if r >= 0:
            ev[r][1].record(stream)
        st.backward(0, dy, dx)
        if r >= 0:
            ev[r][2].record(stream)
        st.step(0.0, 0.0)      # clears the accumulated gradients; parameters unchanged
    torch.cuda.synchronize()
    tf = float(np.median([e[0].elapsed_time(e[1]) for e in ev]))
    tb = float(np.median([e[1].elapsed_time(e[2]) for e in ev]))
    st.close()
    return tf, tb


def unit_memory(sub, bmax, shape, dtype, layout, grad_in, out_bytes=0.0):
    """(act_l, w_l, fixed_l) of a unit for the planner's memory check, Eq. (3) plus a fixed term:
    (2 + 1) w_l + K * beta * act_l + fixed_l.  w_l = fp32 parameter bytes.  Eq. (3) has no term for the
    workspace (activation gradients, reduction partials: independent of K, growing with beta in steps) or
    for the derived weight copies; both are fitted here as fixed_l + beta * (part of act_l) from what
    asteroid_stage_plan_memory reports at beta = 1, 2, 4, ... and bmax: act_l is the slope between beta = 1
    and bmax of stash + workspace, fixed_l the largest amount by which any of those batch sizes lies above
    that line, plus the copies.  out_bytes (a_l, the unit's output per sample) is added to act_l: a unit
    measured alone writes its output gradient into the caller's buffer, inside a longer stage that buffer
    is part of the stage's workspace.  Charging the workspace slope once per stashed micro-batch
    over-states it for K > 1: the check errs on the safe side, never below what the library reports.
    No GPU needed."""
    grid = sorted({bmax} | {b for b in (1 << i for i in range(31)) if b < bmax})
    rows = {b: A.plan_memory(sub, b, 1, 1, shape, dtype, layout, grad_in) for b in grid}
    mod, opt, _, _ = rows[bmax]
    T = {b: rows[b][2] + rows[b][3] for b in grid}
    slope = (T[bmax] - T[1]) / (bmax - 1) if bmax > 1 else 0.0
    slope = max(slope, max(rows[b][2] / b for b in grid))      # never below the stash alone
    fixed = max(0.0, max(T[b] - slope * b for b in grid)) + max(0, mod - 2 * opt)
    return slope + out_bytes, opt, fixed


def profile_model(layers, in_shape, dtype, layout, betas, needs_input_grad=False, reps=20, log=None):
    """Tables of a model: list of units, each {lo, hi, kinds, a, act, w, tf{beta}, tb{beta}};
    a, act in bytes per sample, w in bytes, times in ms."""
    esz = 2 if dtype == "bf16" else 4
    units, shape = [], tuple(in_shape)
    bmax = max(betas)
    for lo, hi in split_units(layers):
        sub = layers[lo:hi]
        out = _out_shape(sub, shape)
        grad_in = needs_input_grad or lo > 0
        a_l = int(np.prod(out)) * (4 if sub[-1]["kind"] == "softmax_ce" else esz)
        act_l, w_l, fixed_l = unit_memory(sub, bmax, shape, dtype, layout, grad_in, a_l)
        u = dict(lo=lo, hi=hi, kinds=[L["kind"] for L in sub], in_shape=list(shape), out_shape=list(out),
                 a=a_l, act=act_l, w=w_l, fixed=fixed_l, tf={}, tb={})
        for beta in betas:
            tf, tb = time_unit(sub, shape, beta, dtype, layout, grad_in, reps=reps)
            u["tf"][beta], u["tb"][beta] = tf, tb
            if log:
                print("unit %3d-%3d beta %4d  tf %8.4f ms  tb %8.4f ms" % (lo, hi, beta, tf, tb), file=log, flush=True)
        units.append(u)
        shape = out
    return units


def tables_for_planner(units, B, n_devices=1):
    """tf, tb [n_devices][L][B+1] (piecewise linear between the measured batch sizes, 0 at 0,
    the last slope beyond the largest one), a, act, w, fixed [L]: the planner's input for a pool of
    identical devices."""
    L = len(units)
    tf = np.zeros((n_devices, L, B + 1))
    tb = np.zeros((n_devices, L, B + 1))
    grid = np.arange(B + 1, dtype=np.float64)
    for l, u in enumerate(units):
        bs = sorted(int(b) for b in u["tf"])
        for name, dst in (("tf", tf), ("tb", tb)):
            t = {int(k): v for k, v in u[name].items()}
            xs = [0.0] + [float(b) for b in bs]
            ys = [0.0] + [t[b] for b in bs]
            v = np.interp(grid, xs, ys)
            if B > bs[-1] and len(bs) > 1:
                slope = (t[bs[-1]] - t[bs[-2]]) / (bs[-1] - bs[-2])
                over = grid > bs[-1]
                v[over] = t[bs[-1]] + slope * (grid[over] - bs[-1])
            dst[:, l, :] = v
    a = np.array([u["a"] for u in units], dtype=np.float64)
    act = np.array([u["act"] for u in units], dtype=np.float64)
    w = np.array([u["w"] for u in units], dtype=np.float64)
    fixed = np.array([u.get("fixed", 0.0) for u in units], dtype=np.float64)
    return tf, tb, a, act, w, fixed


def markdown(units, betas, title):
    """The tables as text: one row per unit, then the whole model and its time per sample."""
    out = ["# " + title, "",
           "a_l = output bytes per sample, act_l = activation memory per sample, w_l = fp32 parameter bytes; "
           "t_f / t_b in microseconds per call at batch size beta.", ""]
    head = "| layers | unit | a_l KB | act_l KB | w_l KB | " + " | ".join("t_f(%d)" % b for b in betas) + " | " + \
        " | ".join("t_b(%d)" % b for b in betas) + " |"
    out += [head, "|" + "---|" * (5 + 2 * len(betas))]
    for u in units:
        name = "+".join(k.replace("batchnorm2d", "bn").replace("conv2d", "conv").replace("layernorm", "ln")
                        for k in u["kinds"] if k not in ("res_begin",))
        if len(name) > 40:
            name = name[:37] + "..."
        out.append("| %d-%d | %s | %.1f | %.1f | %.1f | " % (u["lo"], u["hi"] - 1, name, u["a"] / 1024,
                                                            u["act"] / 1024, u["w"] / 1024) +
                   " | ".join("%.0f" % (1e3 * u["tf"][b]) for b in betas) + " | " +
                   " | ".join("%.0f" % (1e3 * u["tb"][b]) for b in betas) + " |")
    tot_f = {b: sum(u["tf"][b] for u in units) for b in betas}
    tot_b = {b: sum(u["tb"][b] for u in units) for b in betas}
    out.append("| all | sum over units | | %.1f | %.1f | " % (sum(u["act"] for u in units) / 1024,
                                                            sum(u["w"] for u in units) / 1024) +
               " | ".join("%.0f" % (1e3 * tot_f[b]) for b in betas) + " | " +
               " | ".join("%.0f" % (1e3 * tot_b[b]) for b in betas) + " |")
    out.append("| all | per sample | | | | " + " | ".join("%.1f" % (1e3 * tot_f[b] / b) for b in betas) + " | " +
               " | ".join("%.1f" % (1e3 * tot_b[b] / b) for b in betas) + " |")
    return "\n".join(out) + "\n"


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--betas", default="1,2,4,8,16,32")
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--out", default=None, help="write the tables as JSON")
    ap.add_argument("--plan-devices", type=int, default=0,
                    help="also plan this many identical devices with the measured tables")
    ap.add_argument("--plan-B", type=int, default=32)
    ap.add_argument("--plan-M", type=int, default=8)
    ap.add_argument("--link-gbs", type=float, default=153.0, help="device-to-device bandwidth, GB/s")
    ap.add_argument("--budget-gb", type=float, default=288.0, help="memory budget per device, GB")
    args = ap.parse_args(argv)
    from asteroid_workloads import get_config
    cfg = get_config(args.workload)
    betas = [int(b) for b in args.betas.split(",")]
    units = profile_model(cfg.layers, cfg.in_shape, cfg.dtype, cfg.layout, betas, cfg.needs_input_grad,
                          reps=args.reps, log=sys.stderr)
    text = markdown(units, betas, "%s (%s, %s %s): profiler tables measured through the C ABI" % (
        args.workload, cfg.name, cfg.dtype, cfg.layout))
    if args.plan_devices > 0:
        import time
        from . import planner as PL
        N, B, M = args.plan_devices, args.plan_B, args.plan_M
        tf, tb, a, act, w, fixed = tables_for_planner(units, B, N)
        bw = np.full((N, N), args.link_gbs * 1e6)          # bytes per millisecond
        u = np.full(N, args.budget_gb * 1e9)
        pr = PL.Problem(tf, tb, a, act, w, u, bw, B, M, block=max(1, B // 16), fixed=fixed)
        t0 = time.perf_counter()
        lat, stages, y = PL.plan_hpp(pr)
        dt = time.perf_counter() - t0
        one = PL.allocate(pr, 0, len(units), [0], 1)
        text += "\nPlan for %d identical devices, %g GB each, %g GB/s links, B = %d, M = %d (Alg. 2, %.1f ms of " \
                "planning over %d units):\n\n" % (N, args.budget_gb, args.link_gbs, B, M, dt * 1e3, len(units))
        for k, (lo, hi, G) in enumerate(stages):
            text += "- stage %d: units %d-%d (layers %d-%d) on devices %s, samples per micro-batch %s\n" % (
                k, lo, hi - 1, units[lo]["lo"], units[hi - 1]["hi"] - 1, G, [y[d] for d in G])
        text += "\nEstimated HPP-Round latency (Eq. (4)) %.3f ms = %.0f samples/s; one device alone: %.3f ms = " \
                "%.0f samples/s.\n" % (lat, B * M / lat * 1e3, M * (one[1] + one[2]), B / (one[1] + one[2]) * 1e3)
    print(text)
    if args.out:
        with open(args.out, "w") as f:
            json.dump(dict(workload=args.workload, betas=betas, units=units), f, indent=1)


if __name__ == "__main__":
    main()
