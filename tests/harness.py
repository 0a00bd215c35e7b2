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
    st = OracleStage(cfg.layers, cfg.B, cfg.M, cfg.in_shape, cfg.layout, cfg.needs_input_grad)
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


def run_hip(cfg, inp, K=1, rounds=2, debug_layers=None):
    """Returns the per-round results of the HIP stage (numpy fp32) and, if asked, the
    activations of `debug_layers` for micro-batch 0 of round 0."""
    import torch
    import paper_2408_08015_amd as A
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    st = A.Stage(cfg.layers, cfg.B, cfg.M, K, cfg.in_shape, cfg.dtype, cfg.layout, cfg.needs_input_grad,
                 stream=torch.cuda.current_stream().cuda_stream)
    st.set_params(inp["params"])
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
    losses = torch.zeros(M, device=dev, dtype=torch.float32)
    res, dbg = [], {}

    def fwd(m, r):
        sl = slice(m * B, (m + 1) * B)
        st.forward(m, x[sl], labels[sl] if labels is not None else None, y[sl],
                   losses[m:m + 1] if cfg.loss_tail else None)
        if debug_layers and r == 0 and m == 0:
            for li in debug_layers:
                try:
                    dbg[li] = st.debug_activation(0, li)
                except A.AsteroidError:
                    pass

    for r in range(rounds):
        for m in range(min(K, M)):
            fwd(m, r)
        for m in range(M):
            sl = slice(m * B, (m + 1) * B)
            st.backward(m, dy[sl] if dy is not None else None, dx[sl] if dx is not None else None)
            if m + K < M:
                fwd(m + K, r)
        torch.cuda.synchronize()
        G = st.get_grads()
        st.step(cfg.lr, cfg.momentum)
        torch.cuda.synchronize()
        res.append(dict(y=y.float().cpu().numpy(), loss=float(losses.sum().item()) if cfg.loss_tail else None,
                        dx=dx.float().cpu().numpy() if dx is not None else None, G=G, W=st.get_params()))
    mem = st.memory()
    st.close()
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
        out["r%d.G" % r] = max(gw, key=lambda t: t[1])
        out["r%d.W" % r] = max(ww, key=lambda t: t[1])
        out["r%d.G_all" % r] = gw
    return out
