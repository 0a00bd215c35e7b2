"""Drives the HIP stage and the CPU oracle through the same 1F1B call sequence on the same
seeded inputs and scores the difference (rel-L2 per tensor)."""
import numpy as np

from asteroid_workloads import gen


def rel_l2(a, b):
    """||a-b|| / ||b|| with b the oracle; tiny references fall back to an absolute bound."""
    a = np.asarray(a, np.float64).ravel()
    b = np.asarray(b, np.float64).ravel()
    nb = np.linalg.norm(b)
    if nb < 1e-30:
        return 0.0 if np.linalg.norm(a) <= 1e-6 * np.sqrt(max(a.size, 1)) else float("inf")
    return float(np.linalg.norm(a - b) / nb)


def split_params(layers, flat):
    out, off = [], 0
    for (li, name, shape, _, _) in gen.param_specs(layers):
        n = int(np.prod(shape))
        out.append(("L%d.%s" % (li, name), flat[off:off + n]))
        off += n
    return out


def run_oracle(cfg, inp, K=1, rounds=2, keep_acts=False):
    from oracle import OracleStage, run_round
    st = OracleStage(cfg.layers, cfg.B, cfg.M, cfg.in_shape, cfg.layout, cfg.needs_input_grad,
                     storage="bf16" if cfg.dtype == "bf16" else "f64")
    st.keep_acts = keep_acts
    st.set_params(inp["params"])
    target = inp["labels"] if cfg.loss_tail else inp["dy"]
    res = []
    for _ in range(rounds):
        ys, loss, dxs = run_round(st, inp["x"], target, K=K)
        G = st.G.copy()
        st.step(cfg.lr, cfg.momentum)
        res.append(dict(y=np.concatenate(ys), loss=loss,
                        dx=np.concatenate(dxs) if cfg.needs_input_grad else None, G=G, W=st.W.copy()))
    return res, st


def run_hip(cfg, inp, K=1, rounds=2, debug_layers=None, static_backward=False, forward_stream=False):
    """Returns the per-round results of the HIP stage (numpy fp32) and, if asked, the
    activations of `debug_layers` for micro-batch 0 of round 0.  static_backward: the backward
    passes go through asteroid_stage_backward_static.  forward_stream: the forward passes run on
    a second stream (asteroid_stage_set_forward_stream)."""
    import torch
    import paper_2408_08015_amd as A
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    st = A.Stage(cfg.layers, cfg.B, cfg.M, K, cfg.in_shape, cfg.dtype, cfg.layout, cfg.needs_input_grad,
                 stream=torch.cuda.current_stream().cuda_stream)
    st.set_params(inp["params"])
    fs = None
    if forward_stream:
        fs = A.stream_create()
        st.set_forward_stream(fs)
    x = torch.from_numpy(inp["x"]).to(dev).to(tdt).contiguous()
    B, M = cfg.B, cfg.M
    if cfg.loss_tail:
        labels = torch.from_numpy(inp["labels"]).to(dev)
        ncls = gen.out_shape(cfg.layers, cfg.in_shape)[0]
        y = torch.zeros((B * M, ncls), device=dev, dtype=torch.float32)
        dy = None
    else:
        labels = None
        dy = torch.from_numpy(inp["dy"]).to(dev).to(tdt).contiguous()
        y = torch.zeros_like(dy)
    dx = torch.zeros_like(x) if cfg.needs_input_grad else None
    losses = torch.zeros(M * 4, device=dev, dtype=torch.float32)
    res, dbg = [], {}
    # one separately allocated (hence aligned) buffer per micro-batch, as a pipeline would hold
    mbs = lambda t: None if t is None else [t[m * B:(m + 1) * B].clone() for m in range(M)]
    xs, ys, dys, dxs, labs = mbs(x), mbs(y), mbs(dy), mbs(dx), mbs(labels)

    def fwd(m, r):
        st.forward(m, xs[m], labs[m] if labs is not None else None, ys[m],
                   losses[4 * m:4 * m + 1] if cfg.loss_tail else None)
        if debug_layers and r == 0 and m == 0:
            for li in debug_layers:
                try:
                    dbg[li] = st.debug_activation(0, li)
                except A.AsteroidError:
                    pass

    torch.cuda.synchronize()  # the inputs exist before either stream reads them
    for r in range(rounds):
        for m in range(min(K, M)):
            fwd(m, r)
        for m in range(M):
            (st.backward_static if static_backward else st.backward)(
                m, dys[m] if dys is not None else None, dxs[m] if dxs is not None else None)
            if m + K < M:
                fwd(m + K, r)
        torch.cuda.synchronize()
        G = st.get_grads()
        st.step(cfg.lr, cfg.momentum)
        torch.cuda.synchronize()
        res.append(dict(y=torch.cat(ys).float().cpu().numpy(),
                        loss=float(losses.double().sum().item()) if cfg.loss_tail else None,
                        dx=torch.cat(dxs).float().cpu().numpy() if dxs is not None else None, G=G,
                        W=st.get_params()))
    mem = st.memory()
    st.close()
    if fs:
        A.stream_destroy(fs)
    return res, dbg, mem


def score(cfg, hip, ora):
    """dict of rel-L2 errors: y, dx, loss, worst G tensor, worst W tensor per round."""
    out = {}
    for r, (h, o) in enumerate(zip(hip, ora)):
        out["r%d.y" % r] = rel_l2(h["y"], o["y"])
        if cfg.needs_input_grad:
            out["r%d.dx" % r] = rel_l2(h["dx"], o["dx"])
        if cfg.loss_tail:
            out["r%d.loss" % r] = abs(h["loss"] - o["loss"]) / abs(o["loss"])
        gw = [(n, rel_l2(a, b)) for (n, a), (_, b) in zip(split_params(cfg.layers, h["G"]), split_params(cfg.layers, o["G"]))]
        ww = [(n, rel_l2(a, b)) for (n, a), (_, b) in zip(split_params(cfg.layers, h["W"]), split_params(cfg.layers, o["W"]))]
        out["r%d.G" % r] = max(gw, key=lambda t: t[1], default=("-", 0.0))   # no parameters: nothing to score
        out["r%d.W" % r] = max(ww, key=lambda t: t[1], default=("-", 0.0))
        out["r%d.G_all" % r] = gw
    return out


# ---------------------------------------------------------------- stored expected values
def golden_path(name):
    import os
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "%s_full.npz" % name)


def golden_velocity(cfg, n):
    """The seeded initial velocity used by tests/golden/make_golden.py."""
    rng = np.random.Generator(np.random.PCG64(cfg.seed + 7))
    return (rng.standard_normal(n) * 0.05).astype(np.float32)


def run_hip_one_round(cfg, inp, v0=None, K=1, forward_stream=False):
    """One HPP-Round on the GPU at the launch configurations bench.py times (K = 1 on one stream; K = 3
    with the forward passes on a second stream).  Returns y, loss, dx, G (before the update), W (after
    it) as numpy arrays."""
    import torch
    import paper_2408_08015_amd as A
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    st = A.Stage(cfg.layers, cfg.B, cfg.M, K, cfg.in_shape, cfg.dtype, cfg.layout, cfg.needs_input_grad,
                 stream=torch.cuda.current_stream().cuda_stream)
    st.set_params(inp["params"])
    if v0 is not None:
        st.set_velocity(v0)
    fs = None
    if forward_stream:
        fs = A.stream_create()
        st.set_forward_stream(fs)
    x = torch.from_numpy(inp["x"]).to(dev).to(tdt).contiguous()
    B, M = cfg.B, cfg.M
    if cfg.loss_tail:
        labels = torch.from_numpy(inp["labels"]).to(dev)
        y = torch.zeros((B * M, gen.out_shape(cfg.layers, cfg.in_shape)[0]), device=dev)
        dy = None
    else:
        labels = None
        dy = torch.from_numpy(inp["dy"]).to(dev).to(tdt).contiguous()
        y = torch.zeros_like(dy)
    dx = torch.zeros_like(x) if cfg.needs_input_grad else None
    losses = torch.zeros(M * 4, device=dev)
    mbs = lambda t: None if t is None else [t[m * B:(m + 1) * B].clone() for m in range(M)]
    xs, ys, dys, dxs, labs = mbs(x), mbs(y), mbs(dy), mbs(dx), mbs(labels)

    def fwd(m):
        st.forward(m, xs[m], labs[m] if labs is not None else None, ys[m],
                   losses[4 * m:4 * m + 1] if cfg.loss_tail else None)

    torch.cuda.synchronize()  # the inputs exist before either stream reads them
    for m in range(min(K, M)):
        fwd(m)
    for m in range(M):
        st.backward(m, dys[m] if dys is not None else None, dxs[m] if dxs is not None else None)
        if m + K < M:
            fwd(m + K)
    torch.cuda.synchronize()
    G = st.get_grads()
    st.step(cfg.lr, cfg.momentum)
    torch.cuda.synchronize()
    out = dict(y=torch.cat(ys).float().cpu().numpy(), loss=float(losses.double().sum().item()),
               dx=torch.cat(dxs).float().cpu().numpy() if dxs is not None else None, G=G, W=st.get_params(),
               V=st.get_velocity())
    st.close()
    if fs:
        A.stream_destroy(fs)
    return out


def grad_error(hv, ov, g_rms):
    """(error, floored): rel-L2 of a parameter tensor's gradient against the oracle's `ov`.  A shift
    (BatchNorm beta, bias) that feeds another BatchNorm through a linear map has a gradient that
    cancels: exactly where the map sends constants to constants (1x1 conv), up to what the zero padding
    of a 3x3 window leaves at the image border otherwise.  Such a tensor has no norm of its own to be
    relative to (fp32 noise of the cancelling sums is of the size of the OTHER gradients): below 1 % of
    the global RMS per entry it is scored against that floor, and reported as floored."""
    ov = np.asarray(ov, np.float64)
    err = np.linalg.norm(np.asarray(hv, np.float64) - ov)
    floor = 1e-2 * g_rms * np.sqrt(ov.size)
    if np.linalg.norm(ov) < floor:
        return float(err / floor), True
    return float(err / np.linalg.norm(ov)), False


def score_golden(cfg, hip, gold):
    """rel-L2 on the stored entries: y, dx (seeded samples: `y`, `dx`; structured sets - tile edges,
    plane borders, first / last entries: `ys`, `dxs`), loss, and per parameter tensor G and W.
    `floored`: the tensors scored by grad_error's floor.  For bf16 configs also the distance to the
    plain fp64 oracle (`f64.*`, reported, not a bar)."""
    out = {"y": rel_l2(hip["y"].ravel()[gold["y_idx"]], gold["y"])}
    if "ys_idx" in gold:
        out["ys"] = rel_l2(hip["y"].ravel()[gold["ys_idx"]], gold["ys"])
    if cfg.needs_input_grad:
        out["dx"] = rel_l2(hip["dx"].ravel()[gold["dx_idx"]], gold["dx"])
        if "dxs_idx" in gold:
            out["dxs"] = rel_l2(hip["dx"].ravel()[gold["dxs_idx"]], gold["dxs"])
    if cfg.loss_tail:
        out["loss"] = abs(hip["loss"] - float(gold["loss"])) / abs(float(gold["loss"]))
    g_rms = float(gold["G_rms"])
    gs, ws, floored, gs64 = [], [], [], []
    for name, hv in split_params(cfg.layers, hip["G"]):
        idx = gold["idx/" + name]
        e, fl = grad_error(hv[idx], gold["G/" + name], g_rms)
        gs.append((name, e))
        if fl:
            floored.append(name)
        if "f64/G/" + name in gold:
            gs64.append((name, grad_error(hv[idx], gold["f64/G/" + name], g_rms)[0]))
    for name, hv in split_params(cfg.layers, hip["W"]):
        idx = gold["idx/" + name]
        ws.append((name, rel_l2(hv[idx], gold["W/" + name])))
    out["G"] = max(gs, key=lambda t: t[1])
    out["W"] = max(ws, key=lambda t: t[1])
    out["G_all"] = gs
    out["G_median"] = float(np.median([e for _, e in gs]))
    out["floored"] = floored
    if "f64/y" in gold:
        out["f64.y"] = rel_l2(hip["y"].ravel()[gold["y_idx"]], gold["f64/y"])
        if cfg.needs_input_grad:
            out["f64.dx"] = rel_l2(hip["dx"].ravel()[gold["dx_idx"]], gold["f64/dx"])
        out["f64.G"] = max(gs64, key=lambda t: t[1])
        out["f64.G_median"] = float(np.median([e for _, e in gs64]))
    return out
