"""Seeded input generators: activations, labels / upstream gradients, parameters.

Draw order for a config with seed s, from numpy Generator(PCG64(s)):
x (boundary layout), then labels or dy, then the parameters in flat order.
Flat parameter order = layer order; inside a layer weight then bias
(BatchNorm / LayerNorm: gamma then beta; MHA: W_qkv[3D][D], b_qkv[3D], W_o[D][D], b_o[D]).
Conv weights are logically [Cout][Cin/groups][kh][kw], linear weights [out][in].
"""
import numpy as np


def param_specs(layers):
    """List of (layer_index, name, shape, fan_in, role) in flat order.
    role: "weight" (random init), "bias" (zero), "gamma" (one), "beta" (zero)."""
    specs = []
    for i, L in enumerate(layers):
        k = L["kind"]
        if k == "conv2d":
            cg = L["cin"] // L["groups"]
            specs.append((i, "weight", (L["cout"], cg, L["k"], L["k"]), cg * L["k"] * L["k"], "weight"))
            if L["bias"]:
                specs.append((i, "bias", (L["cout"],), 0, "bias"))
        elif k == "linear":
            specs.append((i, "weight", (L["cout"], L["cin"]), L["cin"], "weight"))
            if L["bias"]:
                specs.append((i, "bias", (L["cout"],), 0, "bias"))
        elif k == "batchnorm2d":
            specs.append((i, "gamma", (L["c"],), 0, "gamma"))
            specs.append((i, "beta", (L["c"],), 0, "beta"))
        elif k == "layernorm":
            specs.append((i, "gamma", (L["d"],), 0, "gamma"))
            specs.append((i, "beta", (L["d"],), 0, "beta"))
        elif k == "mha":
            d = L["d"]
            specs.append((i, "w_qkv", (3 * d, d), d, "weight"))
            specs.append((i, "b_qkv", (3 * d,), 0, "bias"))
            specs.append((i, "w_o", (d, d), d, "weight"))
            specs.append((i, "b_o", (d,), 0, "bias"))
    return specs


def num_params(layers):
    return int(sum(int(np.prod(s[2])) for s in param_specs(layers)))


def round_to_bf16(a):
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(a.shape)


def make_params(layers, rng, init="kaiming", randomize_affine=False):
    """Flat fp32 parameter vector.  kaiming: N(0, 2/fan_in); normal0.02: N(0, 0.02^2).
    Biases 0, gamma 1, beta 0 unless randomize_affine (then small random values, so
    unit tests exercise those terms)."""
    parts = []
    for (_, _, shape, fan_in, role) in param_specs(layers):
        n = int(np.prod(shape))
        if role == "weight":
            std = np.sqrt(2.0 / fan_in) if init == "kaiming" else 0.02
            p = rng.standard_normal(n) * std
        elif role == "gamma":
            p = rng.uniform(0.5, 1.5, n) if randomize_affine else np.ones(n)
        else:
            p = rng.standard_normal(n) * 0.1 if randomize_affine else np.zeros(n)
        parts.append(p.astype(np.float32))
    return np.concatenate(parts) if parts else np.zeros(0, np.float32)


def boundary_shape(layout, per_sample, n):
    if layout == "nchw" or layout == "bsd":
        return (n,) + tuple(per_sample)
    if layout == "nhwc":
        c, h, w = per_sample
        return (n, h, w, c)
    raise ValueError(layout)


def layer_shapes(layers, in_shape):
    """Per-sample logical output shape of every layer ((C,H,W), (S,D) or (classes,))."""
    s = tuple(in_shape)
    se = []
    res = []
    shapes = []
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
            ho = (h + 2 * L["pad"] - L["k"]) // L["stride"] + 1
            wo = (w + 2 * L["pad"] - L["k"]) // L["stride"] + 1
            s = (L["cout"], ho, wo)
        elif k == "maxpool2x2":
            s = (s[0], s[1] // 2, s[2] // 2)
        elif k == "maxpool3x3s2":
            s = (s[0], (s[1] - 1) // 2 + 1, (s[2] - 1) // 2 + 1)
        elif k == "global_avgpool":
            s = (s[0],)
        elif k == "linear":
            s = s[:-1] + (L["cout"],)
        shapes.append(s)
    return shapes


def out_shape(layers, in_shape):
    """Per-sample logical output shape of the stage."""
    shapes = layer_shapes(layers, in_shape)
    return shapes[-1] if shapes else tuple(in_shape)


def make_inputs(cfg, randomize_affine=False):
    """dict(x, labels | dy, params) for a StageConfig.  x, dy are fp32 arrays in the
    boundary layout covering all M*B samples; in bf16 configs they are already rounded
    to bf16-representable values so every consumer sees identical numbers."""
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    n = cfg.B * cfg.M
    x = rng.standard_normal(boundary_shape(cfg.layout, cfg.in_shape, n)).astype(np.float32)
    out = dict()
    if cfg.loss_tail:
        ncls = out_shape(cfg.layers, cfg.in_shape)[0]
        out["labels"] = rng.integers(0, ncls, size=n).astype(np.int32)
    else:
        osh = out_shape(cfg.layers, cfg.in_shape)
        dy = rng.standard_normal(boundary_shape(cfg.layout, osh, n)).astype(np.float32)
        out["dy"] = round_to_bf16(dy) if cfg.dtype == "bf16" else dy
    out["x"] = round_to_bf16(x) if cfg.dtype == "bf16" else x
    out["params"] = make_params(cfg.layers, rng, cfg.init, randomize_affine)
    return out
