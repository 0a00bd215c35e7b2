"""CPU fp64 oracle: one pipeline stage's training step.  TEST INFRASTRUCTURE ONLY.

Follows Sec. 3.2: a device holds a stage model (consecutive layers), runs the
forward pass and backward pass per micro-batch, accumulates gradients over the M
micro-batches of a mini-batch, and applies them once per HPP-Round.  Activations
stashed by a forward are released by the matching backward (1F1B, Sec. 3.2).

Readings where the paper is silent (the optimiser, loss scaling, BatchNorm scope)
are those of the repository's design notes: momentum SGD v = mu*v + G,
W = W - lr*v, G = 0; a loss tail divides by M*B so G is the gradient of the
mini-batch mean loss; a stage fed an upstream gradient applies no scaling;
BatchNorm statistics are those of the micro-batch.

Stages whose tensors are bf16 ("bf16 compute, fp32 accumulation, fp32 master
weights"): with storage="bf16" the oracle applies exactly the roundings that this
arithmetic type prescribes and nothing else -- the weight matrices are rounded to bf16
when used as operands (the fp32 master copy is what the update changes), and every
layer's output activation is rounded to bf16 (round-to-nearest-even); all sums stay in
fp64 and rounding passes gradients through unchanged.  This puts the decisions that a
float comparison takes (ReLU masks, max-pool arg-max) in the kernel's precision on both
sides, which a comparison of a bf16 stage needs: a pure fp64 run picks a different
arg-max wherever two window entries agree to 8 bits.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this.
It imports nothing from the HIP package.
"""
import numpy as np

from . import layers as L

F = np.float64


def round_bf16(a):
    """fp64 -> nearest fp32 -> nearest bf16 (ties to even), returned as fp64."""
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    u = a32.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(a32.shape).astype(F)


def _param_shapes(layer):
    k = layer["kind"]
    if k == "conv2d":
        s = [(layer["cout"], layer["cin"] // layer["groups"], layer["k"], layer["k"])]
        return s + ([(layer["cout"],)] if layer["bias"] else [])
    if k == "linear":
        s = [(layer["cout"], layer["cin"])]
        return s + ([(layer["cout"],)] if layer["bias"] else [])
    if k == "batchnorm2d":
        return [(layer["c"],), (layer["c"],)]
    if k == "layernorm":
        return [(layer["d"],), (layer["d"],)]
    if k == "mha":
        d = layer["d"]
        return [(3 * d, d), (3 * d,), (d, d), (d,)]
    return []


class OracleStage:
    """Same logical calls as the C ABI (create / forward / backward / step), on host fp64."""

    def __init__(self, layers, B, M, in_shape, layout="nchw", needs_input_grad=True, storage="f64"):
        assert storage in ("f64", "bf16")
        self.storage = storage
        self.layers = [dict(l) for l in layers]
        self.B, self.M = B, M
        self.in_shape = tuple(in_shape)
        self.layout = layout
        self.needs_input_grad = needs_input_grad
        self.shapes = [_param_shapes(l) for l in self.layers]
        self.offsets = []
        off = 0
        for shp in self.shapes:
            o = []
            for s in shp:
                o.append(off)
                off += int(np.prod(s))
            self.offsets.append(o)
        self.nparams = off
        self.W = np.zeros(off, F)
        self.Wop = self.W
        self.G = np.zeros(off, F)
        self.V = np.zeros(off, F)
        self.stash = {}
        self.keep_acts = False     # tests may ask for every layer's output (logical layout)
        self.acts = {}
        self.loss_tail = self.layers[-1]["kind"] == "softmax_ce"
        # BatchNorm running statistics (tracked, never scored)
        self.running = {i: [np.zeros(l["c"], F), np.ones(l["c"], F)]
                        for i, l in enumerate(self.layers) if l["kind"] == "batchnorm2d"}

    # ---- parameters
    def set_params(self, flat):
        assert flat.size == self.nparams
        self.W = np.asarray(flat, F).copy()
        self._refresh_operands()

    def _refresh_operands(self):
        """Weights as the layers see them: the master copy, or (bf16 storage) its weight
        matrices rounded to bf16; biases and normalisation parameters stay as they are."""
        if self.storage != "bf16":
            self.Wop = self.W
            return
        self.Wop = self.W.copy()
        for i, l in enumerate(self.layers):
            mats = {"conv2d": [0], "linear": [0], "mha": [0, 2]}.get(l["kind"], [])
            for t in mats:
                o, n = self.offsets[i][t], int(np.prod(self.shapes[i][t]))
                self.Wop[o:o + n] = round_bf16(self.W[o:o + n])

    def set_velocity(self, flat):
        self.V = np.asarray(flat, F).copy()

    def _p(self, vec, i):
        return [vec[o:o + int(np.prod(s))].reshape(s) for o, s in zip(self.offsets[i], self.shapes[i])]

    def _acc(self, i, grads):
        """In-place accumulation G += grad_m (Sec. 3.2)."""
        for o, s, g in zip(self.offsets[i], self.shapes[i], grads):
            self.G[o:o + g.size] += g.ravel()

    # ---- layout at the boundary
    def _to_logical(self, a):
        a = np.asarray(a, F)
        return a.transpose(0, 3, 1, 2) if (self.layout == "nhwc" and a.ndim == 4) else a

    def _to_boundary(self, a):
        return np.ascontiguousarray(a.transpose(0, 2, 3, 1)) if (self.layout == "nhwc" and a.ndim == 4) else a

    # ---- forward pass of micro-batch mb
    def forward(self, mb, x, labels=None):
        assert mb not in self.stash
        a = self._to_logical(x)
        saved = []
        res = []
        se = []
        loss = None
        logits = None
        trace = []
        for i, l in enumerate(self.layers):
            if i > 0 and self.keep_acts:
                trace.append(a)
            k = l["kind"]
            P = self._p(self.Wop, i)
            if k == "conv2d":
                saved.append(a)
                a = L.conv2d_fwd(a, P[0], P[1] if l["bias"] else None, l["stride"], l["pad"], l["groups"])
            elif k == "batchnorm2d":
                a, (xhat, istd, mu, var) = L.batchnorm2d_fwd(a, P[0], P[1], l["eps"])
                saved.append((xhat, istd))
                n = xhat.size // xhat.shape[1]
                rm, rv = self.running[i]
                rm += 0.1 * (mu - rm)
                rv += 0.1 * (var * n / max(n - 1, 1) - rv)
            elif k == "layernorm":
                a, sv = L.layernorm_fwd(a, P[0], P[1], l["eps"])
                saved.append(sv)
            elif k == "relu":
                saved.append(a)
                a = L.relu_fwd(a)
            elif k == "relu6":
                saved.append(a)
                a = L.relu6_fwd(a)
            elif k == "gelu":
                saved.append(a)
                a = L.gelu_fwd(a)
            elif k == "swish":
                saved.append(a)
                a = L.swish_fwd(a)
            elif k == "sigmoid":
                saved.append(a)
                a = L.sigmoid_fwd(a)
            elif k == "se_begin":
                # squeeze-and-excitation: the layers up to se_scale turn this tensor into one
                # gate per sample and channel, which then scales it
                se.append(a)
                saved.append(None)
            elif k == "se_scale":
                xs = se.pop()
                saved.append((xs, a))
                a = xs * a[:, :, None, None]
            elif k == "res_begin":
                res.append(a)
                saved.append(None)
            elif k == "res_swap":
                # two-branch residual block (a ResNet block whose shortcut has layers of its own):
                # the main branch ends here; the layers up to res_add run on the block's input
                a, res[-1] = res[-1], a
                saved.append(None)
            elif k == "res_add":
                a = a + res.pop()
                saved.append(None)
            elif k == "global_avgpool":
                saved.append(a.shape)
                a = L.global_avgpool_fwd(a)
            elif k == "maxpool2x2":
                y, idx = L.maxpool2x2_fwd(a)
                saved.append((idx, a.shape))
                a = y
            elif k == "maxpool3x3s2":
                y, idx = L.maxpool3x3s2_fwd(a)
                saved.append((idx, a.shape))
                a = y
            elif k == "linear":
                saved.append(a)
                a = L.linear_fwd(a, P[0], P[1] if l["bias"] else None)
            elif k == "mha":
                y, sv = L.mha_fwd(a, P[0], P[1], P[2], P[3], l["heads"])
                saved.append((a, sv))
                a = y
            elif k == "softmax_ce":
                logits = a
                loss, p = L.softmax_ce_fwd(a, np.asarray(labels), self.M * self.B)
                saved.append((p, np.asarray(labels)))
            else:
                raise ValueError(k)
            if self.storage == "bf16" and k not in ("softmax_ce", "res_begin", "res_swap", "se_begin"):
                a = round_bf16(a)
        self.stash[mb] = saved
        if self.keep_acts:
            trace.append(a)
            self.acts[mb] = trace          # trace[i] = output of layer i
        if self.loss_tail:
            return logits, loss
        return self._to_boundary(a), None

    # ---- backward pass of micro-batch mb
    def backward(self, mb, dy=None):
        saved = self.stash.pop(mb)            # the backward releases the stash
        g = None if self.loss_tail else self._to_logical(dy)
        skip = []
        for i in range(len(self.layers) - 1, -1, -1):
            l = self.layers[i]
            k = l["kind"]
            P = self._p(self.Wop, i)
            sv = saved[i]
            if k == "softmax_ce":
                g = L.softmax_ce_bwd(sv[0], sv[1], self.M * self.B)
            elif k == "conv2d":
                g, grads = L.conv2d_bwd(sv, P[0], g, l["stride"], l["pad"], l["groups"], l["bias"])
                self._acc(i, grads)
            elif k == "batchnorm2d":
                g, grads = L.batchnorm2d_bwd(g, P[0], sv[0], sv[1])
                self._acc(i, grads)
            elif k == "layernorm":
                g, grads = L.layernorm_bwd(g, P[0], sv[0], sv[1])
                self._acc(i, grads)
            elif k == "relu":
                g = L.relu_bwd(g, sv)
            elif k == "relu6":
                g = L.relu6_bwd(g, sv)
            elif k == "gelu":
                g = L.gelu_bwd(g, sv)
            elif k == "swish":
                g = L.swish_bwd(g, sv)
            elif k == "sigmoid":
                g = L.sigmoid_bwd(g, sv)
            elif k == "se_scale":
                xs, gate = sv
                skip.append(g * gate[:, :, None, None])      # through the scaled tensor
                g = (g * xs).sum(axis=(2, 3))                # through the gate
            elif k == "se_begin":
                g = g + skip.pop()
            elif k == "res_add":
                skip.append(g)
            elif k == "res_swap":
                # g is the gradient of the block's input through the shortcut branch; the main
                # branch's output gets the gradient res_add set aside
                g, skip[-1] = skip[-1], g
            elif k == "res_begin":
                g = g + skip.pop()
            elif k == "global_avgpool":
                g = L.global_avgpool_bwd(g, sv[2], sv[3])
            elif k == "maxpool2x2":
                g = L.maxpool2x2_bwd(g, sv[0], sv[1][2], sv[1][3])
            elif k == "maxpool3x3s2":
                g = L.maxpool3x3s2_bwd(g, sv[0], sv[1][2], sv[1][3])
            elif k == "linear":
                g, grads = L.linear_bwd(sv, P[0], g, l["bias"])
                self._acc(i, grads)
            elif k == "mha":
                g, grads = L.mha_bwd(sv[0], P[0], P[2], g, sv[1], l["heads"])
                self._acc(i, grads)
        return self._to_boundary(g) if self.needs_input_grad else None

    # ---- weight update, once per HPP-Round
    def step(self, lr, momentum):
        assert not self.stash
        self.V = momentum * self.V + self.G
        self.W = self.W - lr * self.V
        self._refresh_operands()
        self.G = np.zeros_like(self.G)


def run_round(stage, x, target, K=1):
    """One HPP-Round in 1F1B order with K warm-up forwards: returns per-micro-batch
    outputs, the summed loss (loss-tailed stages) and per-micro-batch input grads."""
    M, B = stage.M, stage.B
    ys, dxs, loss = [None] * M, [None] * M, 0.0

    def fwd(m):
        xm = x[m * B:(m + 1) * B]
        if stage.loss_tail:
            y, l = stage.forward(m, xm, target[m * B:(m + 1) * B])
            return y, l
        return stage.forward(m, xm)

    for m in range(min(K, M)):
        ys[m], l = fwd(m)
        loss += l or 0.0
    for m in range(M):
        dxs[m] = stage.backward(m, None if stage.loss_tail else target[m * B:(m + 1) * B])
        if m + K < M:
            ys[m + K], l = fwd(m + K)
            loss += l or 0.0
    return ys, loss, dxs
