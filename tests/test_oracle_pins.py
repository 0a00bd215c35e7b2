"""Pins of the CPU oracle against things other than itself: brute force, finite
differences, adjoint identities, closed forms, invariants, and an independent
library's float64 autograd (PyTorch CPU) on the same layers."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

from asteroid_workloads import configs as C
from asteroid_workloads import gen
from oracle import OracleStage, run_round
from oracle import layers as L

RNG = lambda s: np.random.Generator(np.random.PCG64(s))


# ----------------------------------------------------------------- brute force conv
def brute_conv(x, w, b, stride, pad, groups):
    n, cin, h, wd = x.shape
    cout, cg, k, _ = w.shape
    og = cout // groups
    ho = (h + 2 * pad - k) // stride + 1
    wo = (wd + 2 * pad - k) // stride + 1
    y = np.zeros((n, cout, ho, wo))
    for nn in range(n):
        for o in range(cout):
            g = o // og
            for i in range(ho):
                for j in range(wo):
                    acc = b[o] if b is not None else 0.0
                    for c in range(cg):
                        for u in range(k):
                            for v in range(k):
                                ii, jj = i * stride - pad + u, j * stride - pad + v
                                if 0 <= ii < h and 0 <= jj < wd:
                                    acc += w[o, c, u, v] * x[nn, g * cg + c, ii, jj]
                    y[nn, o, i, j] = acc
    return y


@pytest.mark.parametrize("cin,cout,k,stride,pad,groups,h,w", [
    (3, 4, 3, 1, 1, 1, 5, 7), (4, 6, 3, 2, 1, 1, 7, 5), (4, 4, 3, 2, 1, 4, 6, 7),
    (6, 6, 3, 1, 1, 6, 5, 5), (5, 3, 1, 1, 0, 1, 4, 3), (4, 8, 3, 1, 1, 2, 5, 4),
    (2, 2, 5, 1, 2, 2, 7, 7),
])
def test_conv_brute_force(cin, cout, k, stride, pad, groups, h, w):
    r = RNG(1)
    x = r.standard_normal((2, cin, h, w))
    wt = r.standard_normal((cout, cin // groups, k, k))
    b = r.standard_normal(cout)
    y = L.conv2d_fwd(x, wt, b, stride, pad, groups)
    np.testing.assert_allclose(y, brute_conv(x, wt, b, stride, pad, groups), rtol=1e-12, atol=1e-12)


def test_conv_adjoint_identities():
    r = RNG(2)
    for (cin, cout, k, s, p, g, h, w) in [(6, 8, 3, 2, 1, 1, 9, 7), (8, 8, 3, 1, 1, 8, 6, 6), (8, 4, 1, 1, 0, 1, 5, 5)]:
        x = r.standard_normal((3, cin, h, w))
        wt = r.standard_normal((cout, cin // g, k, k))
        y = L.conv2d_fwd(x, wt, None, s, p, g)
        gy = r.standard_normal(y.shape)
        dx, (dw,) = L.conv2d_bwd(x, wt, gy, s, p, g, False)
        lhs = (y * gy).sum()
        assert abs(lhs - (x * dx).sum()) < 1e-10 * abs(lhs) + 1e-10
        assert abs(lhs - (wt * dw).sum()) < 1e-10 * abs(lhs) + 1e-10


def test_depthwise_equals_block_diagonal_dense():
    r = RNG(3)
    c = 5
    x = r.standard_normal((2, c, 6, 7))
    wd = r.standard_normal((c, 1, 3, 3))
    dense = np.zeros((c, c, 3, 3))
    for i in range(c):
        dense[i, i] = wd[i, 0]
    np.testing.assert_allclose(L.conv2d_fwd(x, wd, None, 2, 1, c), L.conv2d_fwd(x, dense, None, 2, 1, 1), atol=1e-13)


def test_pointwise_is_per_pixel_matvec():
    r = RNG(4)
    x = r.standard_normal((2, 5, 3, 4))
    w = r.standard_normal((7, 5, 1, 1))
    y = L.conv2d_fwd(x, w, None, 1, 0, 1)
    for n in range(2):
        for i in range(3):
            for j in range(4):
                np.testing.assert_allclose(y[n, :, i, j], w[:, :, 0, 0] @ x[n, :, i, j], atol=1e-13)


# ----------------------------------------------------------------- finite differences
def fd_check(f, args, idx, gy, analytic, h=1e-6, tol=1e-6, samples=40, seed=0):
    """Central differences of L = <gy, f(args)> w.r.t. args[idx] at random coordinates."""
    r = RNG(seed)
    a = args[idx]
    flat = a.reshape(-1)
    for _ in range(min(samples, flat.size)):
        j = r.integers(flat.size)
        old = flat[j]
        flat[j] = old + h
        fp = (f(*args) * gy).sum()
        flat[j] = old - h
        fm = (f(*args) * gy).sum()
        flat[j] = old
        num = (fp - fm) / (2 * h)
        ana = analytic.reshape(-1)[j]
        assert abs(num - ana) <= tol * max(1.0, abs(ana)), (j, num, ana)


def test_fd_conv():
    r = RNG(5)
    for (cin, cout, k, s, p, g) in [(4, 6, 3, 2, 1, 1), (6, 6, 3, 1, 1, 6), (4, 6, 1, 1, 0, 1), (6, 6, 3, 2, 1, 6)]:
        x = r.standard_normal((2, cin, 6, 5))
        w = r.standard_normal((cout, cin // g, k, k))
        b = r.standard_normal(cout)
        f = lambda x, w, b: L.conv2d_fwd(x, w, b, s, p, g)
        gy = r.standard_normal(f(x, w, b).shape)
        dx, (dw, db) = L.conv2d_bwd(x, w, gy, s, p, g, True)
        fd_check(f, [x, w, b], 0, gy, dx)
        fd_check(f, [x, w, b], 1, gy, dw)
        fd_check(f, [x, w, b], 2, gy, db)


def test_fd_batchnorm_layernorm():
    r = RNG(6)
    x = r.standard_normal((3, 4, 5, 5)) * 2 + 1
    ga, be = r.uniform(0.5, 1.5, 4), r.standard_normal(4)
    f = lambda x, ga, be: L.batchnorm2d_fwd(x, ga, be, 1e-5)[0]
    y, (xhat, istd, _, _) = L.batchnorm2d_fwd(x, ga, be, 1e-5)
    gy = r.standard_normal(y.shape)
    dx, (dga, dbe) = L.batchnorm2d_bwd(gy, ga, xhat, istd)
    fd_check(f, [x, ga, be], 0, gy, dx)
    fd_check(f, [x, ga, be], 1, gy, dga)
    fd_check(f, [x, ga, be], 2, gy, dbe)
    x = r.standard_normal((2, 5, 16)) * 2 + 1
    ga, be = r.uniform(0.5, 1.5, 16), r.standard_normal(16)
    f = lambda x, ga, be: L.layernorm_fwd(x, ga, be, 1e-5)[0]
    y, (xhat, istd) = L.layernorm_fwd(x, ga, be, 1e-5)
    gy = r.standard_normal(y.shape)
    dx, (dga, dbe) = L.layernorm_bwd(gy, ga, xhat, istd)
    fd_check(f, [x, ga, be], 0, gy, dx)
    fd_check(f, [x, ga, be], 1, gy, dga)
    fd_check(f, [x, ga, be], 2, gy, dbe)


def test_fd_pointwise_and_pool():
    r = RNG(7)
    x = r.standard_normal((2, 3, 6, 6)) * 4
    x[np.abs(x) < 1e-3] = 0.5
    x[np.abs(x - 6) < 1e-3] = 5.0
    gy = r.standard_normal(x.shape)
    fd_check(L.relu_fwd, [x], 0, gy, L.relu_bwd(gy, x))
    fd_check(L.relu6_fwd, [x], 0, gy, L.relu6_bwd(gy, x))
    fd_check(L.gelu_fwd, [x], 0, gy, L.gelu_bwd(gy, x))
    fd_check(L.swish_fwd, [x], 0, gy, L.swish_bwd(gy, x))
    fd_check(L.sigmoid_fwd, [x], 0, gy, L.sigmoid_bwd(gy, x))
    y, idx = L.maxpool2x2_fwd(x)
    gp = r.standard_normal(y.shape)
    fd_check(lambda x: L.maxpool2x2_fwd(x)[0], [x], 0, gp, L.maxpool2x2_bwd(gp, idx, 6, 6))
    ga = r.standard_normal((2, 3))
    fd_check(L.global_avgpool_fwd, [x], 0, ga, L.global_avgpool_bwd(ga, 6, 6))


def test_fd_linear_softmax_mha():
    r = RNG(8)
    x = r.standard_normal((4, 6))
    w = r.standard_normal((5, 6))
    b = r.standard_normal(5)
    gy = r.standard_normal((4, 5))
    dx, (dw, db) = L.linear_bwd(x, w, gy, True)
    fd_check(L.linear_fwd, [x, w, b], 0, gy, dx)
    fd_check(L.linear_fwd, [x, w, b], 1, gy, dw)
    fd_check(L.linear_fwd, [x, w, b], 2, gy, db)
    lab = np.array([0, 3, 4, 1])
    loss, p = L.softmax_ce_fwd(x, lab, 8.0)
    dz = L.softmax_ce_bwd(p, lab, 8.0)
    fd_check(lambda z: np.array(L.softmax_ce_fwd(z, lab, 8.0)[0]), [x], 0, np.array(1.0), dz)
    d, heads = 8, 2
    x = r.standard_normal((2, 5, d))
    wq, bq = r.standard_normal((3 * d, d)) * 0.5, r.standard_normal(3 * d) * 0.1
    wo, bo = r.standard_normal((d, d)) * 0.5, r.standard_normal(d) * 0.1
    f = lambda x, wq, bq, wo, bo: L.mha_fwd(x, wq, bq, wo, bo, heads)[0]
    y, sv = L.mha_fwd(x, wq, bq, wo, bo, heads)
    gy = r.standard_normal(y.shape)
    dx, grads = L.mha_bwd(x, wq, wo, gy, sv, heads)
    args = [x, wq, bq, wo, bo]
    for i, a in enumerate([dx] + grads):
        fd_check(f, args, i, gy, a)


# ----------------------------------------------------------------- closed forms / invariants
def test_gelu_matches_math_erf():
    xs = np.linspace(-4, 4, 41)
    ref = np.array([x * 0.5 * (1 + math.erf(x / math.sqrt(2))) for x in xs])
    np.testing.assert_allclose(L.gelu_fwd(xs), ref, atol=1e-14)
    assert abs(L.gelu_fwd(np.array([1.0]))[0] - 0.8413447460685429) < 1e-14      # Phi(1)


def test_sigmoid_swish_closed_forms():
    xs = np.linspace(-6, 6, 25)
    ref = np.array([1.0 / (1.0 + math.exp(-x)) for x in xs])
    np.testing.assert_allclose(L.sigmoid_fwd(xs), ref, atol=1e-15)
    np.testing.assert_allclose(L.sigmoid_fwd(xs) + L.sigmoid_fwd(-xs), 1.0, atol=1e-15)   # s(-x) = 1 - s(x)
    np.testing.assert_allclose(L.sigmoid_fwd(xs), 0.5 * (1.0 + np.tanh(xs / 2.0)), atol=1e-15)
    np.testing.assert_allclose(L.swish_fwd(xs) - L.swish_fwd(-xs), xs, atol=1e-14)        # odd part is x/2 * 2
    assert L.swish_fwd(np.array([0.0]))[0] == 0.0
    assert abs(L.swish_fwd(np.array([1.0]))[0] - 0.7310585786300049) < 1e-15              # 1/(1+1/e)


def test_squeeze_excite_with_zero_fc_halves_the_tensor():
    """Both SE linear layers at zero: the gate is sigmoid(0) = 1/2 for every channel, the block
    scales its input by 1/2, passes half the gradient through and gives the FC weights none
    except through the last bias."""
    Ls = C.squeeze_excite(6, 2)
    cfg = C.StageConfig("se", Ls, 2, 1, (6, 5, 5), "f32", "nchw", True, 3)
    st = OracleStage(cfg.layers, cfg.B, cfg.M, cfg.in_shape)
    st.set_params(np.zeros(st.nparams))
    r = RNG(5)
    x = r.standard_normal((2, 6, 5, 5))
    dy = r.standard_normal((2, 6, 5, 5))
    y, _ = st.forward(0, x)
    np.testing.assert_allclose(y, 0.5 * x, atol=1e-15)
    dx = st.backward(0, dy)
    np.testing.assert_allclose(dx, 0.5 * dy, atol=1e-15)
    gW1, gb1, gW2, gb2 = st._p(st.G, 2) + st._p(st.G, 4)
    assert not gW1.any() and not gb1.any() and not gW2.any()
    # d gate = sum_hw dy*x per (sample, channel); sigmoid'(0) = 1/4; the bias sums over samples
    np.testing.assert_allclose(gb2, 0.25 * (dy * x).sum(axis=(0, 2, 3)), atol=1e-13)


def test_bn_ln_invariants():
    r = RNG(9)
    x = r.standard_normal((4, 3, 5, 5)) * 3 + 2
    ga, be = r.uniform(0.5, 1.5, 3), r.standard_normal(3)
    y, (xhat, istd, mu, var) = L.batchnorm2d_fwd(x, ga, be, 1e-5)
    np.testing.assert_allclose(y.mean(axis=(0, 2, 3)), be, atol=1e-12)
    np.testing.assert_allclose(y.var(axis=(0, 2, 3)), ga ** 2 * var / (var + 1e-5), rtol=1e-12)
    np.testing.assert_allclose(var, x.var(axis=(0, 2, 3)), rtol=1e-12)
    g = r.standard_normal(x.shape)
    _, (xhat, istd, _, _) = L.batchnorm2d_fwd(x, ga, be, 0.0)     # sum xhat^2 = n exactly when eps = 0
    dx, _ = L.batchnorm2d_bwd(g, ga, xhat, istd)
    np.testing.assert_allclose(dx.sum(axis=(0, 2, 3)), 0, atol=1e-11)
    np.testing.assert_allclose((dx * xhat).sum(axis=(0, 2, 3)), 0, atol=1e-10)
    dx2, _ = L.batchnorm2d_bwd(g + 3.7, ga, xhat, istd)
    np.testing.assert_allclose(dx, dx2, atol=1e-11)
    x = r.standard_normal((3, 4, 32))
    ga, be = r.uniform(0.5, 1.5, 32), r.standard_normal(32)
    y, (xhat, istd) = L.layernorm_fwd(x, ga, be, 0.0)
    g = r.standard_normal(x.shape)
    dx, _ = L.layernorm_bwd(g, ga, xhat, istd)
    np.testing.assert_allclose(dx.sum(axis=-1), 0, atol=1e-11)
    np.testing.assert_allclose((dx * xhat).sum(axis=-1), 0, atol=1e-11)


def test_softmax_pool_attention_closed_forms():
    r = RNG(10)
    z = r.standard_normal((5, 10))
    lab = r.integers(0, 10, 5)
    loss, p = L.softmax_ce_fwd(z, lab, 5)
    np.testing.assert_allclose(p.sum(axis=1), 1, atol=1e-14)
    np.testing.assert_allclose(L.softmax_ce_bwd(p, lab, 5).sum(axis=1), 0, atol=1e-14)
    loss0, _ = L.softmax_ce_fwd(np.zeros((5, 10)), lab, 5)
    assert abs(loss0 - math.log(10)) < 1e-14
    x = r.standard_normal((2, 3, 6, 8))
    y, idx = L.maxpool2x2_fwd(x)
    g = r.standard_normal(y.shape)
    assert abs(L.maxpool2x2_bwd(g, idx, 6, 8).sum() - g.sum()) < 1e-12
    # ties go to the first element in row-major order
    yt, it = L.maxpool2x2_fwd(np.zeros((1, 1, 2, 2)))
    assert it[0, 0, 0, 0] == 0
    # W_q = 0 -> uniform attention -> every head output is the sequence mean of V
    d, heads, s = 8, 2, 6
    xs = r.standard_normal((2, s, d))
    wq = r.standard_normal((3 * d, d))
    wq[:d] = 0
    bq = np.zeros(3 * d)
    y, (q, k, v, p, oc) = L.mha_fwd(xs, wq, bq, np.eye(d), np.zeros(d), heads)
    np.testing.assert_allclose(p, 1.0 / s, atol=1e-15)
    vfull = xs @ wq[2 * d:].T
    np.testing.assert_allclose(y, np.broadcast_to(vfull.mean(axis=1, keepdims=True), y.shape), atol=1e-13)


# ----------------------------------------------------------------- whole-stage pins
def tiny_stage(cfg):
    st = OracleStage(cfg.layers, cfg.B, cfg.M, cfg.in_shape, cfg.layout, cfg.needs_input_grad)
    inp = gen.make_inputs(cfg, randomize_affine=True)
    st.set_params(inp["params"])
    return st, inp


def test_zero_fc_gives_log_classes_and_zero_projection_is_identity():
    cfg = C.cfg1(B=2, M=2, hw=4)
    st, inp = tiny_stage(cfg)
    W = st.W.copy()
    fc = [i for i, l in enumerate(cfg.layers) if l["kind"] == "linear"][0]
    o = st.offsets[fc]
    W[o[0]:] = 0.0
    st.set_params(W)
    _, loss, _ = run_round(st, inp["x"], inp["labels"])
    assert abs(loss - math.log(10)) < 1e-13
    # a residual block whose last BatchNorm has gamma = beta = 0 returns its input
    blk = C.irb(8, 8, 1, 6)
    s2 = OracleStage(blk, 2, 1, (8, 5, 5))
    p = gen.make_params(blk, RNG(3))
    last_bn = [i for i, l in enumerate(blk) if l["kind"] == "batchnorm2d"][-1]
    p[s2.offsets[last_bn][0]:s2.offsets[last_bn][0] + 16] = 0
    s2.set_params(p)
    x = RNG(4).standard_normal((2, 8, 5, 5))
    y, _ = s2.forward(0, x)
    np.testing.assert_allclose(y, x, atol=1e-14)


def test_fd_whole_cfg1_stage():
    """Central differences of the summed CE loss of a tiny cfg-1 stage w.r.t. parameters and input."""
    cfg = C.cfg1(B=2, M=2, hw=4)
    st, inp = tiny_stage(cfg)
    x = inp["x"].astype(np.float64)
    _, loss, dxs = run_round(st, x, inp["labels"])
    G = st.G.copy()
    dx = np.concatenate(dxs)
    W0 = st.W.copy()

    def loss_at(W, xx):
        s = OracleStage(cfg.layers, cfg.B, cfg.M, cfg.in_shape)
        s.set_params(W)
        return run_round(s, xx, inp["labels"])[1]

    r = RNG(11)
    h = 1e-6
    for j in r.integers(0, W0.size, 60):
        Wp, Wm = W0.copy(), W0.copy()
        Wp[j] += h
        Wm[j] -= h
        num = (loss_at(Wp, x) - loss_at(Wm, x)) / (2 * h)
        assert abs(num - G[j]) <= 2e-6 * max(1.0, abs(G[j])), (j, num, G[j])
    for j in r.integers(0, x.size, 20):
        xp, xm = x.copy(), x.copy()
        xp.reshape(-1)[j] += h
        xm.reshape(-1)[j] -= h
        num = (loss_at(W0, xp) - loss_at(W0, xm)) / (2 * h)
        assert abs(num - dx.reshape(-1)[j]) <= 2e-6 * max(1.0, abs(dx.reshape(-1)[j]))


@pytest.mark.parametrize("cfg", [C.cfg4(B=2, M=3, hw=6, cin=4, c=6), C.cfg5(B=2, M=3, S=5, d=16, heads=2, ffn=32, nlayers=2)])
def test_microbatch_sum_equals_whole_batch_for_bn_free(cfg):
    st, inp = tiny_stage(cfg)
    run_round(st, inp["x"], inp["dy"])
    whole = OracleStage(cfg.layers, cfg.B * cfg.M, 1, cfg.in_shape, cfg.layout)
    whole.set_params(inp["params"])
    run_round(whole, inp["x"], inp["dy"])
    np.testing.assert_allclose(st.G, whole.G, rtol=1e-11, atol=1e-12)


def test_result_independent_of_K_and_sgd_closed_form():
    cfg = C.cfg2(B=2, M=4, hw=8)
    outs = []
    for K in (1, 3, 4):
        st, inp = tiny_stage(cfg)
        ys, _, dxs = run_round(st, inp["x"], inp["dy"], K=K)
        outs.append((np.concatenate(ys), np.concatenate(dxs), st.G.copy()))
    for o in outs[1:]:
        for a, b in zip(outs[0], o):
            assert np.array_equal(a, b)
    G, W0 = st.G.copy(), st.W.copy()
    st.step(0.01, 0.9)
    np.testing.assert_allclose(st.W, W0 - 0.01 * G, atol=1e-15)
    assert not st.G.any()
    st.G = G.copy()                      # an identical second round's gradient
    st.step(0.01, 0.9)
    np.testing.assert_allclose(st.W, W0 - 0.01 * G - 0.01 * 1.9 * G, atol=1e-15)


def test_two_branch_residual_is_the_sum_of_its_branches():
    """res_begin, main, res_swap, shortcut, res_add against the two branches run as stages of
    their own on the same input: outputs add, input gradients add, parameter gradients are those
    of the branches."""
    main = [C.conv(6, 10, 3, 2, 1), C.bn(10), C.simple("relu")]
    short = [C.conv(6, 10, 1, 2), C.bn(10)]
    block = [C.simple("res_begin")] + main + [C.simple("res_swap")] + short + [C.simple("res_add")]
    r = RNG(12)
    x = r.standard_normal((2, 6, 7, 7))
    dy = r.standard_normal((2, 10, 4, 4))
    stages = {name: OracleStage(L, 2, 1, (6, 7, 7)) for name, L in (("block", block), ("main", main), ("short", short))}
    wm = RNG(3).standard_normal(stages["main"].nparams)
    ws = RNG(4).standard_normal(stages["short"].nparams)
    res = {}
    for name, w in (("main", wm), ("short", ws), ("block", np.concatenate([wm, ws]))):
        st = stages[name]
        st.set_params(w)
        y, _ = st.forward(0, x)
        dx = st.backward(0, dy)
        res[name] = (y, dx, st.G.copy())
    np.testing.assert_allclose(res["block"][0], res["main"][0] + res["short"][0], atol=1e-12)
    np.testing.assert_allclose(res["block"][1], res["main"][1] + res["short"][1], atol=1e-12)
    np.testing.assert_allclose(res["block"][2], np.concatenate([res["main"][2], res["short"][2]]), atol=1e-12)


def test_maxpool3x3s2_brute_force_and_ties():
    r = RNG(21)
    for h, w in ((7, 7), (8, 6), (1, 1), (2, 5)):
        x = r.standard_normal((2, 3, h, w))
        y, idx = L.maxpool3x3s2_fwd(x)
        ho, wo = (h - 1) // 2 + 1, (w - 1) // 2 + 1
        assert y.shape == (2, 3, ho, wo)
        g = r.standard_normal(y.shape)
        dx = L.maxpool3x3s2_bwd(g, idx, h, w)
        ref_y = np.zeros_like(y)
        ref_dx = np.zeros_like(x)
        for n in range(2):
            for c in range(3):
                for i in range(ho):
                    for j in range(wo):
                        best, arg = -np.inf, None
                        for u in range(3):
                            for v in range(3):
                                ii, jj = 2 * i - 1 + u, 2 * j - 1 + v
                                if 0 <= ii < h and 0 <= jj < w and x[n, c, ii, jj] > best:
                                    best, arg = x[n, c, ii, jj], (ii, jj)
                        ref_y[n, c, i, j] = best
                        ref_dx[n, c, arg[0], arg[1]] += g[n, c, i, j]
        np.testing.assert_array_equal(y, ref_y)
        np.testing.assert_allclose(dx, ref_dx, atol=1e-15)
    # all equal (a ReLU output of zeros): the gradient goes to the first in-image position of each window
    z = np.zeros((1, 1, 4, 4))
    y, idx = L.maxpool3x3s2_fwd(z)
    dx = L.maxpool3x3s2_bwd(np.ones((1, 1, 2, 2)), idx, 4, 4)
    expect = np.zeros((4, 4))
    expect[0, 0] = expect[0, 1] = expect[1, 0] = expect[1, 1] = 1.0
    np.testing.assert_array_equal(dx[0, 0], expect)


def test_resnet50_schedule():
    """16 bottleneck blocks, 25.56 M parameters with the 1000-way classifier (the published count),
    224 -> 7 spatial, four projection shortcuts."""
    Ls = C.resnet50_layers()
    assert sum(1 for l in Ls if l["kind"] == "res_add") == 16
    assert sum(1 for l in Ls if l["kind"] == "res_swap") == 4
    assert gen.out_shape(Ls[:-3], (3, 224, 224)) == (2048, 7, 7)
    n = gen.num_params(Ls)
    assert abs(n - 25.557e6) < 0.01e6, n


def test_efficientnet_b1_schedule():
    """23 MBConv blocks, 7.8 M parameters with the 1000-way classifier (the published count of
    EfficientNet-B1), 240 -> 8 spatial, every block with its squeeze-and-excitation."""
    L = C.efficientnet_b1_layers()
    assert sum(1 for l in L if l["kind"] == "se_scale") == 23
    assert gen.out_shape(L[:-3], (3, 240, 240)) == (1280, 8, 8)
    n = gen.num_params(L)
    assert abs(n - 7.79e6) < 0.05e6, n
    dws = [l for l in L if l["kind"] == "conv2d" and l["groups"] > 1]
    assert len(dws) == 23 and sum(1 for l in dws if l["k"] == 5) == 12


def test_mobilenetv2_schedule():
    Ls = C.mobilenetv2_layers()
    assert gen.num_params(Ls) == 3504872
    assert sum(1 for l in Ls if l["kind"] == "conv2d" and l["groups"] > 1) == 17
    assert OracleStage(Ls, 1, 1, (3, 224, 224)).nparams == 3504872


# ----------------------------------------------------------------- independent library cross-check
def torch_stage(cfg, params, x, target, dtype=torch.float64, bf16_storage=False, manual_bn=False):
    """The same layer list through PyTorch CPU functional ops + autograd (float64 by default).
    bf16_storage: weight matrices and every layer output pass through the library's own
    bf16 cast (round to nearest even) with a straight-through gradient.
    manual_bn: BatchNorm written out with elementwise operations and reductions in `dtype` (the
    library routine accumulates its statistics in double on the CPU whatever the tensor's type)."""
    t = lambda a: torch.tensor(np.asarray(a, np.float64)).to(dtype)
    rb = (lambda v: v + (v.float().bfloat16().to(dtype) - v).detach()) if bf16_storage else (lambda v: v)
    W = t(params).requires_grad_(True)
    xs = t(x).requires_grad_(True)
    off = 0

    def take(shape):
        nonlocal off
        n = int(np.prod(shape))
        v = W[off:off + n].reshape(shape)
        off += n
        return v

    total = 0.0
    outs = []
    B, M = cfg.B, cfg.M
    for m in range(M):
        off = 0
        a = xs[m * B:(m + 1) * B]
        if cfg.layout == "nhwc":
            a = a.permute(0, 3, 1, 2)
        res = []
        se = []
        for l in cfg.layers:
            k = l["kind"]
            if k == "conv2d":
                w = rb(take((l["cout"], l["cin"] // l["groups"], l["k"], l["k"])))
                b = take((l["cout"],)) if l["bias"] else None
                a = TF.conv2d(a, w, b, l["stride"], l["pad"], 1, l["groups"])
            elif k == "batchnorm2d":
                ga, be = take((l["c"],)), take((l["c"],))
                if manual_bn:
                    mu = a.mean(dim=(0, 2, 3), keepdim=True)
                    var = ((a - mu) ** 2).mean(dim=(0, 2, 3), keepdim=True)
                    a = (a - mu) / torch.sqrt(var + l["eps"]) * ga[None, :, None, None] + be[None, :, None, None]
                else:
                    a = TF.batch_norm(a, None, None, ga, be, True, 0.1, l["eps"])
            elif k == "layernorm":
                ga, be = take((l["d"],)), take((l["d"],))
                a = TF.layer_norm(a, (l["d"],), ga, be, l["eps"])
            elif k == "relu":
                a = TF.relu(a)
            elif k == "relu6":
                a = TF.relu6(a)
            elif k == "gelu":
                a = TF.gelu(a)
            elif k == "swish":
                a = TF.silu(a)
            elif k == "sigmoid":
                a = torch.sigmoid(a)
            elif k == "se_begin":
                se.append(a)
            elif k == "se_scale":
                a = se.pop() * a[:, :, None, None]
            elif k == "res_begin":
                res.append(a)
            elif k == "res_swap":
                a, res[-1] = res[-1], a
            elif k == "res_add":
                a = a + res.pop()
            elif k == "global_avgpool":
                a = a.mean(dim=(2, 3))
            elif k == "maxpool2x2":
                a = TF.max_pool2d(a, 2, 2)
            elif k == "maxpool3x3s2":
                a = TF.max_pool2d(a, 3, 2, 1)
            elif k == "linear":
                w = rb(take((l["cout"], l["cin"])))
                b = take((l["cout"],)) if l["bias"] else None
                a = TF.linear(a, w, b)
            elif k == "mha":
                d = l["d"]
                wq, bq, wo, bo = rb(take((3 * d, d))), take((3 * d,)), rb(take((d, d))), take((d,))
                at = a.transpose(0, 1)        # (S, N, D)
                o, _ = TF.multi_head_attention_forward(
                    at, at, at, d, l["heads"], wq, bq, None, None, False, 0.0, wo, bo,
                    training=True, need_weights=False)
                a = o.transpose(0, 1)
            elif k == "softmax_ce":
                lab = torch.tensor(target[m * B:(m + 1) * B].astype(np.int64))
                total = total + TF.cross_entropy(a, lab, reduction="sum") / (M * B)
            if k not in ("softmax_ce", "res_begin", "res_swap", "se_begin"):
                a = rb(a)
        if not cfg.loss_tail:
            if cfg.layout == "nhwc":
                a = a.permute(0, 2, 3, 1)
            total = total + (a * t(target[m * B:(m + 1) * B])).sum()
        outs.append(a.detach().numpy())
    total.backward()
    return outs, W.grad.double().numpy(), xs.grad.double().numpy(), float(total.detach())


@pytest.mark.parametrize("cfg", [
    C.cfg1(B=3, M=2, hw=6),
    C.cfg2(B=3, M=2, hw=9),
    C.cfg3(B=3, M=2, hw=64, num_classes=7),
    C.cfg4(B=2, M=2, hw=6, cin=4, c=6),
    C.cfg5(B=2, M=2, S=7, d=16, heads=2, ffn=24, nlayers=2),
    C.cfg6(B=3, M=2, hw=10),
    C.cfg7(B=3, M=2, hw=7, cin=8, mid=4, blocks=2),
    C.StageConfig("stem_pool", [C.conv(3, 8, 7, 2, 3), C.bn(8), C.simple("relu"), C.simple("maxpool3x3s2")], 2, 2, (3, 17, 15), "f32", "nchw", True, 33),
    C.StageConfig("strided_bottlenecks", C.bottleneck(8, 4, 2) + C.bottleneck(16, 4), 3, 2, (8, 9, 9), "f32", "nchw", True, 31),
], ids=lambda c: c.name)
def test_stage_matches_torch_float64_autograd(cfg):
    st, inp = tiny_stage(cfg)
    target = inp["labels"] if cfg.loss_tail else inp["dy"]
    ys, loss, dxs = run_round(st, inp["x"], target)
    t_out, t_G, t_dx, t_loss = torch_stage(cfg, inp["params"], inp["x"], target)
    for a, b in zip(ys, t_out):
        np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-10)
    np.testing.assert_allclose(st.G, t_G, rtol=1e-8, atol=1e-10)
    if cfg.needs_input_grad:
        np.testing.assert_allclose(np.concatenate(dxs), t_dx, rtol=1e-8, atol=1e-10)
    if cfg.loss_tail:
        assert abs(loss - t_loss) < 1e-10


@pytest.mark.parametrize("cfg", [
    C.cfg4(B=2, M=2, hw=6, cin=4, c=6),
    C.cfg5(B=2, M=2, S=7, d=16, heads=2, ffn=24, nlayers=2),
], ids=lambda c: c.name)
def test_bf16_storage_mode_matches_torch_with_library_bf16_casts(cfg):
    """storage="bf16": the prescribed roundings (weight matrices, layer outputs) checked against
    PyTorch float64 autograd with torch's own bfloat16 casts at the same points."""
    inp = gen.make_inputs(cfg, randomize_affine=True)
    st = OracleStage(cfg.layers, cfg.B, cfg.M, cfg.in_shape, cfg.layout, cfg.needs_input_grad, storage="bf16")
    st.set_params(inp["params"])
    ys, _, dxs = run_round(st, inp["x"], inp["dy"])
    t_out, t_G, t_dx, _ = torch_stage(cfg, inp["params"], inp["x"], inp["dy"], bf16_storage=True)
    y = np.concatenate(ys)
    assert np.array_equal(gen.round_to_bf16(y.astype(np.float32)).astype(np.float64), y)   # outputs are bf16 values
    np.testing.assert_allclose(y, np.concatenate(t_out), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(st.G, t_G, rtol=1e-8, atol=1e-10)
    np.testing.assert_allclose(np.concatenate(dxs), t_dx, rtol=1e-8, atol=1e-10)
    # and it is a small perturbation of the unrounded computation
    pure = OracleStage(cfg.layers, cfg.B, cfg.M, cfg.in_shape, cfg.layout, cfg.needs_input_grad)
    pure.set_params(inp["params"])
    yp, _, _ = run_round(pure, inp["x"], inp["dy"])
    assert np.linalg.norm(y - np.concatenate(yp)) <= 2e-2 * np.linalg.norm(np.concatenate(yp))


def test_round_bf16_helper():
    from oracle.stage import round_bf16
    v = np.array([1.0, 1.00390625, 1.01171875, -3.14159, 0.1, 3.0e38])
    r = round_bf16(v)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.015625      # ties go to the even mantissa
    assert r[3] == -3.140625 and abs(r[4] - 0.10009765625) < 1e-15
    assert np.array_equal(round_bf16(r), r)
