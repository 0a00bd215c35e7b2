"""Layer lists and shapes of the benchmark stages.

A stage model is a run of consecutive layers (Sec. 3.2); a mini-batch is split
into M micro-batches of size B.  Micro-batch m holds samples [m*B, (m+1)*B).

Layer dictionaries (keys are plain ints/floats/bools):
  conv2d       cin cout k stride pad groups bias
  batchnorm2d  c eps
  relu / relu6 / gelu / swish / sigmoid / res_begin / res_add / global_avgpool / maxpool2x2 /
  maxpool3x3s2 (3x3 window, stride 2, padding 1) / softmax_ce
  res_swap     inside res_begin ... res_add: ends the main branch; the layers from here to res_add
               form the shortcut branch and run on the tensor res_begin remembered
  se_begin ... se_scale   squeeze-and-excitation: the layers in between (global_avgpool, linear,
               swish, linear, sigmoid) turn the tensor at se_begin into one gate per sample and
               channel; se_scale multiplies that tensor by its gate
  linear       cin cout bias
  layernorm    d eps
  mha          d heads
"""
from dataclasses import dataclass, field
from typing import List, Tuple


def conv(cin, cout, k, stride=1, pad=0, groups=1, bias=False):
    return dict(kind="conv2d", cin=cin, cout=cout, k=k, stride=stride, pad=pad,
                groups=groups, bias=bool(bias))


def bn(c, eps=1e-5):
    return dict(kind="batchnorm2d", c=c, eps=eps)


def simple(kind):
    return dict(kind=kind)


def linear(cin, cout, bias=True):
    return dict(kind="linear", cin=cin, cout=cout, bias=bool(bias))


def irb(cin, cout, stride, expand):
    """MobileNetV2 inverted-residual block: 1x1 expand, BN, ReLU6, 3x3 depthwise,
    BN, ReLU6, 1x1 project, BN, residual add iff stride 1 and cin == cout.
    The expansion conv is absent when expand == 1."""
    hid = cin * expand
    res = stride == 1 and cin == cout
    L = []
    if res:
        L.append(simple("res_begin"))
    if expand != 1:
        L += [conv(cin, hid, 1), bn(hid), simple("relu6")]
    L += [conv(hid, hid, 3, stride, 1, groups=hid), bn(hid), simple("relu6")]
    L += [conv(hid, cout, 1), bn(cout)]
    if res:
        L.append(simple("res_add"))
    return L


def squeeze_excite(c, cr):
    return [simple("se_begin"), simple("global_avgpool"), linear(c, cr), simple("swish"),
            linear(cr, c), simple("sigmoid"), simple("se_scale")]


def mbconv(cin, cout, k, stride, expand, se_ratio=0.25):
    """EfficientNet block: 1x1 expand, BN, swish, kxk depthwise, BN, swish, squeeze-and-excitation
    (reduced to se_ratio * cin channels), 1x1 project, BN, residual add iff stride 1 and
    cin == cout.  The expansion conv is absent when expand == 1."""
    hid = cin * expand
    res = stride == 1 and cin == cout
    L = []
    if res:
        L.append(simple("res_begin"))
    if expand != 1:
        L += [conv(cin, hid, 1), bn(hid), simple("swish")]
    L += [conv(hid, hid, k, stride, k // 2, groups=hid), bn(hid), simple("swish")]
    L += squeeze_excite(hid, max(1, int(cin * se_ratio)))
    L += [conv(hid, cout, 1), bn(cout)]
    if res:
        L.append(simple("res_add"))
    return L


# (t, c, n, s): expansion, output channels, repeats, stride of the first repeat
MBV2_SCHEDULE = [(1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2),
                 (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1)]


def mobilenetv2_layers(num_classes=1000, schedule=MBV2_SCHEDULE, stem=32, last=1280):
    L = [conv(3, stem, 3, 2, 1), bn(stem), simple("relu6")]
    cin = stem
    for t, c, n, s in schedule:
        for i in range(n):
            L += irb(cin, c, s if i == 0 else 1, t)
            cin = c
    L += [conv(cin, last, 1), bn(last), simple("relu6"), simple("global_avgpool"),
          linear(last, num_classes), simple("softmax_ce")]
    return L


# (t, c, n, s, k): expansion, output channels, repeats, stride of the first repeat, depthwise kernel;
# EfficientNet-B0's groups with the repeats scaled by B1's depth factor 1.1 (rounded up)
EFFNET_B1_SCHEDULE = [(1, 16, 2, 1, 3), (6, 24, 3, 2, 3), (6, 40, 3, 2, 5), (6, 80, 4, 2, 3),
                      (6, 112, 4, 1, 5), (6, 192, 5, 2, 5), (6, 320, 2, 1, 3)]


def efficientnet_b1_layers(num_classes=1000, schedule=EFFNET_B1_SCHEDULE, stem=32, last=1280):
    """EfficientNet-B1 (Table 4 workload; width 1.0, depth 1.1, 240x240 input): 3x3 stride-2 stem,
    23 MBConv blocks with squeeze-and-excitation, 1x1 head, pooled classifier."""
    L = [conv(3, stem, 3, 2, 1), bn(stem), simple("swish")]
    cin = stem
    for t, c, n, s, k in schedule:
        for i in range(n):
            L += mbconv(cin, c, k, s if i == 0 else 1, t)
            cin = c
    L += [conv(cin, last, 1), bn(last), simple("swish"), simple("global_avgpool"),
          linear(last, num_classes), simple("softmax_ce")]
    return L


def bottleneck(cin, mid, stride=1):
    """ResNet50 bottleneck block (Table 4 workload): 1x1 reduce, BN, ReLU, 3x3 (carries the stride),
    BN, ReLU, 1x1 expand to 4*mid, BN; shortcut = identity, or 1x1 conv (stride) + BN when the
    shape changes; ReLU after the sum."""
    cout = 4 * mid
    L = [simple("res_begin"),
         conv(cin, mid, 1), bn(mid), simple("relu"),
         conv(mid, mid, 3, stride, 1), bn(mid), simple("relu"),
         conv(mid, cout, 1), bn(cout)]
    if stride != 1 or cin != cout:
        L += [simple("res_swap"), conv(cin, cout, 1, stride), bn(cout)]
    return L + [simple("res_add"), simple("relu")]


# (mid channels, blocks, stride of the first block) of ResNet50's four block groups
RESNET50_SCHEDULE = [(64, 3, 1), (128, 4, 2), (256, 6, 2), (512, 3, 2)]


def resnet50_layers(num_classes=1000, schedule=RESNET50_SCHEDULE, stem=64):
    """ResNet50 (Table 4 workload): 7x7 stride-2 stem, BN, ReLU, 3x3 stride-2 max-pool, 16 bottleneck
    blocks (the stride sits on the 3x3 convolution), pooled classifier."""
    L = [conv(3, stem, 7, 2, 3), bn(stem), simple("relu"), simple("maxpool3x3s2")]
    cin = stem
    for mid, n, s in schedule:
        for i in range(n):
            L += bottleneck(cin, mid, s if i == 0 else 1)
            cin = 4 * mid
    L += [simple("global_avgpool"), linear(cin, num_classes), simple("softmax_ce")]
    return L


def encoder_layer(d, heads, ffn, eps=1e-5):
    """Post-LN encoder layer: h = LN(x + MHA(x)); y = LN(h + W2 GELU(W1 h + b1) + b2)."""
    return [simple("res_begin"), dict(kind="mha", d=d, heads=heads), simple("res_add"),
            dict(kind="layernorm", d=d, eps=eps),
            simple("res_begin"), linear(d, ffn), simple("gelu"), linear(ffn, d),
            simple("res_add"), dict(kind="layernorm", d=d, eps=eps)]


def vgg_layers(cin, c):
    return [conv(cin, c, 3, 1, 1, bias=True), simple("relu"),
            conv(c, c, 3, 1, 1, bias=True), simple("relu"),
            conv(c, c, 3, 1, 1, bias=True), simple("relu"), simple("maxpool2x2")]


@dataclass
class StageConfig:
    name: str
    layers: List[dict]
    B: int
    M: int
    in_shape: Tuple[int, ...]      # per-sample logical shape: (C,H,W) or (S,D)
    dtype: str                     # "f32" | "bf16"  (bf16 = bf16 operands, fp32 accumulate/master)
    layout: str                    # boundary layout: "nchw" | "nhwc" | "bsd"
    needs_input_grad: bool
    seed: int
    lr: float = 0.01
    momentum: float = 0.9
    init: str = "kaiming"          # "kaiming" | "normal0.02"
    note: str = ""

    @property
    def loss_tail(self):
        return self.layers[-1]["kind"] == "softmax_ce"


def cfg1(B=4, M=2, hw=16, seed=1001):
    L = irb(32, 32, 1, 6) + irb(32, 32, 1, 6) + [simple("global_avgpool"), linear(32, 10),
                                               simple("softmax_ce")]
    return StageConfig("cfg1_tiny_cnn", L, B, M, (32, hw, hw), "f32", "nchw", True, seed)


def cfg2(B=32, M=4, hw=56, seed=1002):
    L = irb(24, 32, 2, 6) + irb(32, 32, 1, 6) + irb(32, 32, 1, 6)
    return StageConfig("cfg2_mbv2_stage", L, B, M, (24, hw, hw), "f32", "nchw", True, seed)


def cfg3(B=8, M=8, hw=224, seed=1003, num_classes=1000):
    return StageConfig("cfg3_mbv2_full", mobilenetv2_layers(num_classes), B, M, (3, hw, hw),
                       "f32", "nchw", False, seed)


def cfg4(B=32, M=4, hw=56, cin=128, c=256, seed=1004):
    return StageConfig("cfg4_vgg_bf16", vgg_layers(cin, c), B, M, (cin, hw, hw), "bf16",
                       "nhwc", True, seed)


def cfg5(B=32, M=4, S=128, d=512, heads=8, ffn=2048, nlayers=6, seed=1005):
    L = []
    for _ in range(nlayers):
        L += encoder_layer(d, heads, ffn)
    return StageConfig("cfg5_bert_small_bf16", L, B, M, (S, d), "bf16", "bsd", True, seed,
                       init="normal0.02")


def cfg6(B=32, M=4, hw=60, seed=1006):
    """EfficientNet-B1 (Table 4) third block group at its 240x240 input resolution: three
    MBConv6 blocks with 5x5 depthwise convolutions, 24 -> 40 channels, 60x60 -> 30x30."""
    L = mbconv(24, 40, 5, 2, 6) + mbconv(40, 40, 5, 1, 6) + mbconv(40, 40, 5, 1, 6)
    return StageConfig("cfg6_effnetb1_stage", L, B, M, (24, hw, hw), "f32", "nchw", True, seed)


def cfg7(B=32, M=4, hw=56, seed=1008, cin=64, mid=64, blocks=3):
    """ResNet50's first block group (conv2_x): three bottlenecks, 64 -> 256 channels at 56x56; the
    first one has a projection shortcut."""
    L = []
    c = cin
    for _ in range(blocks):
        L += bottleneck(c, mid)
        c = 4 * mid
    return StageConfig("cfg7_resnet50_stage", L, B, M, (cin, hw, hw), "f32", "nchw", True, seed)


def effnetb1(B=8, M=8, hw=240, seed=1007, num_classes=1000):
    """The whole EfficientNet-B1 as one stage (profiler tables; no stored full-size oracle samples)."""
    return StageConfig("effnetb1_full", efficientnet_b1_layers(num_classes), B, M, (3, hw, hw),
                       "f32", "nchw", False, seed)


def resnet50(B=8, M=8, hw=224, seed=1009, num_classes=1000):
    """The whole ResNet50 as one stage (profiler tables; no stored full-size oracle samples)."""
    return StageConfig("resnet50_full", resnet50_layers(num_classes), B, M, (3, hw, hw), "f32", "nchw",
                       False, seed)


CONFIGS = {
    "cfg1": cfg1, "cfg2": cfg2, "cfg3": cfg3, "cfg4": cfg4, "cfg5": cfg5, "cfg6": cfg6,
    "cfg7": cfg7, "effnetb1": effnetb1, "resnet50": resnet50,
}


def get_config(name, **kw):
    """Full-size config by name ("cfg1".."cfg7"); keyword overrides shrink it for tests."""
    return CONFIGS[name](**kw)
