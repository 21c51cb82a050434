"""Seeded synthetic workloads: layer lists and parameter/input tensors.

This module only *describes* networks and draws random numbers.  It contains
none of the arithmetic of the layers themselves (no convolution, no
normalisation, no pooling, no output-size computation), so that it can feed
both the HIP path and the independent CPU checker with identical data.

Everything is expressed in logical indices: activations ``[N, C, H, W]``,
convolution weights ``[Cout, Cin, R, S]``, linear weights ``[Out, In]``; all
arrays are ``numpy.float32``.  For the bf16 workloads every input and weight
value is rounded to the nearest bf16 number (ties to even) before anybody sees
it, so the stored fp32 values are exactly representable in bf16.

Layer list format (a list of plain dicts, consumed by the binding and by the
checker alike):

``{"kind": "conv", "cout", "kh", "kw", "sh", "sw", "ph", "pw", "bn": bool,
   "act": "none"|"relu", "pool": None | pool-dict, "src": int, "res": int}``
``{"kind": "pool", "pool": pool-dict, "src": int}``
``{"kind": "gap", "src": int}``                       (global average pool)
``{"kind": "linear", "out": int, "act": ..., "src": int}``

``pool-dict = {"kind": "max"|"avg", "kh","kw","sh","sw","ph","pw","count_pad"}``.
``src`` / ``res`` are absolute indices of the layer whose output is consumed;
``src == -1`` means "the previous layer" (the network input for layer 0) and
``res == -1`` means "no residual".

The workloads stand in for the TorchVision CNNs on ``[B, 3, 224, 224]`` inputs
that the paper measures (Sec. V, evaluation set-up): same layer shapes and
sizes, random weights, random inputs.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20031068

# tensor-kind ids used to derive an independent random stream per tensor
_T_INPUT, _T_W, _T_GAMMA, _T_BETA, _T_MEAN, _T_VAR, _T_LABEL, _T_BIAS = range(8)
_T_PRE = 8     # added to _T_GAMMA .. _T_VAR for the input-side BN of a pre-activation convolution


def _rng(seed: int, layer: int, kind: int) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(layer) + 1, int(kind)])


def to_bf16_grid(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 value (ties to even), keep fp32 storage.

    Uses the tensor library's own dtype conversion; no hand-written rounding here.
    """
    import torch

    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def pool_desc(kind="max", k=2, s=2, p=0, count_pad=1):
    return {"kind": kind, "kh": k, "kw": k, "sh": s, "sw": s, "ph": p, "pw": p,
            "count_pad": int(count_pad)}


def conv(cout, k, s=1, p=None, bn=True, act="relu", pool=None, src=-1, res=-1, dw=False, pre_bn=False):
    """dw: depthwise (groups == channels, cout must equal the input channel count; weights [C,1,k,k]).
    pre_bn: a BN + ReLU of the layer's INPUT runs in front of the convolution (pre-activation order)."""
    if p is None:
        p = (k - 1) // 2
    return {"kind": "conv", "cout": cout, "kh": k, "kw": k, "sh": s, "sw": s, "ph": p, "pw": p,
            "bn": bool(bn), "act": act, "pool": pool, "src": src, "res": res, "dw": bool(dw), "pre_bn": bool(pre_bn)}


def pool(kind="max", k=2, s=2, p=0, count_pad=1, src=-1):
    return {"kind": "pool", "pool": pool_desc(kind, k, s, p, count_pad), "src": src}


def concat(src, res):
    """Channel concatenation [layer src | layer res] (absolute layer indices; src = -1: the previous layer)."""
    return {"kind": "concat", "src": src, "res": res}


def gap(src=-1):
    return {"kind": "gap", "src": src}


def linear(out, act="none", src=-1):
    return {"kind": "linear", "out": out, "act": act, "src": src}


# --------------------------------------------------------------------------------------
# network builders
# --------------------------------------------------------------------------------------
def single_block_layers():
    """Config 0: conv3x3 16ch + BN + ReLU + maxpool 2x2 s2."""
    return [conv(16, 3, pool=pool_desc("max", 2, 2, 0))]


def small_cnn_layers():
    """Config 1: 4 fused conv blocks, global average pool, linear 64->10."""
    return [
        conv(32, 3),
        conv(32, 3, pool=pool_desc("max", 2, 2, 0)),
        conv(64, 3),
        conv(64, 3, pool=pool_desc("max", 2, 2, 0)),
        gap(),
        linear(10),
    ]


def mlp_layers(features, depth=3):
    """`depth` linear layers of `features` x `features` with a ReLU between them (the paper's MLP workload,
    Sec. V: three layers, 8192 features)."""
    return [linear(features, act="relu" if i + 1 < depth else "none") for i in range(depth)]


def separable_layers(num_classes=1000, widths=((64, 1), (128, 2), (128, 1), (256, 2), (256, 1), (512, 2), (512, 1), (512, 1),
                                                 (512, 1), (512, 1), (512, 1), (1024, 2), (1024, 1)), stem=32):
    """Config 6: a depthwise-separable chain of the MobileNet kind the paper names for its depthwise rule
    (Sec. III-A): 3x3 stride-2 stem, then per (width, stride) a depthwise 3x3 + BN + ReLU followed by a
    pointwise 1x1 + BN + ReLU, global average pool, linear."""
    L = [conv(stem, 3, s=2)]
    c = stem
    for width, stride in widths:
        L.append(conv(c, 3, s=stride, dw=True))
        L.append(conv(width, 1, p=0))
        c = width
    L.append(gap())
    L.append(linear(num_classes))
    return L


def fire_layers(base, src, squeeze, expand):
    """One fire module appended behind layer `src` (base = index the first new layer will get): 1x1 squeeze + ReLU,
    then a 1x1 and a 3x3 expand + ReLU side by side on the squeezed tensor, joined by channel concatenation."""
    return [conv(squeeze, 1, p=0, bn=False, src=src),
            conv(expand, 1, p=0, bn=False, src=base),
            conv(expand, 3, bn=False, src=base),
            concat(base + 1, base + 2)]


def squeezenet_layers(num_classes=1000):
    """Config 7: a SqueezeNet-1.1-shaped list (one of the evaluation networks of the paper, Sec. VI, where the
    branches of every fire module are joined by a channel concatenation): 3x3 stride-2 stem of 64 filters, then
    max pools (3x3 stride 2, floor mode here) and eight fire modules, a 1x1 classifier convolution + ReLU and a
    global average pool.  No batch norm: bias + ReLU epilogues."""
    L = [conv(64, 3, s=2, p=0, bn=False), pool("max", 3, 2, 0)]
    for group in (((16, 64), (16, 64)), ((32, 128), (32, 128)), ((48, 192), (48, 192), (64, 256), (64, 256))):
        for sq, ex in group:
            L += fire_layers(len(L), len(L) - 1, sq, ex)
        if group[0][0] != 48:
            L.append(pool("max", 3, 2, 0))
    L.append(conv(num_classes, 1, p=0, bn=False))
    L.append(gap())
    return L


def densenet_layers(num_classes=1000, growth=32, blocks=(6, 12, 24, 16), stem=64, bottleneck=4):
    """Config 8: a DenseNet-121-shaped list (one of the evaluation networks of the paper, Sec. VI).  Stem as in the
    ResNet-shaped lists; dense blocks of `blocks[i]` layers, each  BN-ReLU-conv1x1 (bottleneck * growth filters) -
    BN-ReLU-conv3x3 (growth filters)  on the concatenation of the block input and all earlier layers' outputs;
    transitions  BN-ReLU-conv1x1 (half the channels) - 2x2 average pool;  final BN-ReLU, global average pool, linear.
    In list form: the first BN-ReLU of a dense layer is the input-side activation of its 1x1 convolution (pre_bn),
    the second one that convolution's own BN + ReLU; the 3x3 convolution stores its raw output, which the
    concatenation appends; the final BN-ReLU is a 1x1 depthwise convolution with BN + ReLU."""
    L = [conv(stem, 7, s=2, p=3), pool("max", 3, 2, 1)]
    c = stem
    for bi, n in enumerate(blocks):
        feat = len(L) - 1                                      # layer holding the concatenated features so far
        for _ in range(n):
            L.append(conv(bottleneck * growth, 1, p=0, src=feat, pre_bn=True))
            L.append(conv(growth, 3, bn=False, act="none"))
            L.append(concat(feat, len(L) - 1))
            feat = len(L) - 1
            c += growth
        if bi + 1 < len(blocks):
            c //= 2
            L.append(conv(c, 1, p=0, bn=False, act="none", pre_bn=True, pool=pool_desc("avg", 2, 2, 0), src=feat))
    L.append(conv(c, 1, p=0, dw=True))                         # final BN + ReLU
    L.append(gap())
    L.append(linear(num_classes))
    return L


def _stem():
    # conv 7x7 stride 2 pad 3 + BN + ReLU, then max-pool 3x3 stride 2 pad 1
    return [conv(64, 7, s=2, p=3), pool("max", 3, 2, 1)]


def resnet18_layers(num_classes=1000):
    """Configs 2 and 4: stem, 4 stages x 2 basic blocks, gap, linear."""
    L = _stem()
    cin = 64
    for stage, width in enumerate((64, 128, 256, 512)):
        for blk in range(2):
            stride = 2 if (stage > 0 and blk == 0) else 1
            x_idx = len(L) - 1                      # block input
            L.append(conv(width, 3, s=stride, src=x_idx))
            a_idx = len(L) - 1
            if stride != 1 or cin != width:
                L.append(conv(width, 1, s=stride, p=0, act="none", src=x_idx))
                sc_idx = len(L) - 1
            else:
                sc_idx = x_idx
            L.append(conv(width, 3, src=a_idx, res=sc_idx))
            cin = width
    L.append(gap())
    L.append(linear(num_classes))
    return L


def resnet50_layers(num_classes=1000, counts=(3, 4, 6, 3)):
    """Config 3: stem, bottleneck stages [3,4,6,3] (stride on the 3x3), gap, linear."""
    L = _stem()
    cin = 64
    for stage, (width, cnt) in enumerate(zip((64, 128, 256, 512), counts)):
        for blk in range(cnt):
            stride = 2 if (stage > 0 and blk == 0) else 1
            x_idx = len(L) - 1
            L.append(conv(width, 1, p=0, src=x_idx))
            L.append(conv(width, 3, s=stride))
            b_idx = len(L) - 1
            if blk == 0:
                L.append(conv(4 * width, 1, s=stride, p=0, act="none", src=x_idx))
                sc_idx = len(L) - 1
            else:
                sc_idx = x_idx
            L.append(conv(4 * width, 1, p=0, src=b_idx, res=sc_idx))
            cin = 4 * width
    L.append(gap())
    L.append(linear(num_classes))
    return L


# --------------------------------------------------------------------------------------
# parameters and inputs
# --------------------------------------------------------------------------------------
def layer_channels(layers, cin):
    """Output channel count of every layer (channel bookkeeping only)."""
    ch = []
    for i, l in enumerate(layers):
        src = l.get("src", -1)
        c_in = cin if (src == -1 and i == 0) else ch[i - 1 if src == -1 else src]
        if l["kind"] == "conv":
            ch.append(l["cout"])
        elif l["kind"] == "linear":
            ch.append(l["out"])
        elif l["kind"] == "concat":
            ch.append(c_in + ch[l["res"]])
        else:
            ch.append(c_in)
    return ch


def make_params(layers, cin, seed, bf16=False, bias_std=0.0):
    """He-normal weights (std = sqrt(2 / fan_in)), BN gamma U(0.5,1.5), beta U(-0.1,0.1),
    running mean N(0, std 0.1), running var U(0.5,1.5); biases 0 unless bias_std > 0
    (tests use non-zero biases so that a dropped bias term is visible)."""
    ch = layer_channels(layers, cin)
    params = []
    for i, l in enumerate(layers):
        src = l.get("src", -1)
        c_in = cin if (src == -1 and i == 0) else ch[i - 1 if src == -1 else src]
        p = {}
        if l["kind"] == "conv":
            wc_in = 1 if l.get("dw") else c_in            # depthwise: one filter per channel
            fan_in = wc_in * l["kh"] * l["kw"]
            w = _rng(seed, i, _T_W).standard_normal((l["cout"], wc_in, l["kh"], l["kw"]))
            w = (w * np.sqrt(2.0 / fan_in)).astype(np.float32)
            p["w"] = to_bf16_grid(w) if bf16 else w
            b = _rng(seed, i, _T_BIAS).standard_normal(l["cout"]) * bias_std
            p["bias"] = b.astype(np.float32)
            if l["bn"]:
                p["gamma"] = _rng(seed, i, _T_GAMMA).uniform(0.5, 1.5, l["cout"]).astype(np.float32)
                p["beta"] = _rng(seed, i, _T_BETA).uniform(-0.1, 0.1, l["cout"]).astype(np.float32)
                p["mean"] = (_rng(seed, i, _T_MEAN).standard_normal(l["cout"]) * 0.1).astype(np.float32)
                p["var"] = _rng(seed, i, _T_VAR).uniform(0.5, 1.5, l["cout"]).astype(np.float32)
                p["eps"] = 1e-5
            if l.get("pre_bn"):
                p["pre_gamma"] = _rng(seed, i, _T_PRE + _T_GAMMA).uniform(0.5, 1.5, c_in).astype(np.float32)
                p["pre_beta"] = _rng(seed, i, _T_PRE + _T_BETA).uniform(-0.1, 0.1, c_in).astype(np.float32)
                p["pre_mean"] = (_rng(seed, i, _T_PRE + _T_MEAN).standard_normal(c_in) * 0.1).astype(np.float32)
                p["pre_var"] = _rng(seed, i, _T_PRE + _T_VAR).uniform(0.5, 1.5, c_in).astype(np.float32)
                p["eps"] = 1e-5
        elif l["kind"] == "linear":
            w = _rng(seed, i, _T_W).standard_normal((l["out"], c_in))
            w = (w * np.sqrt(2.0 / c_in)).astype(np.float32)
            p["w"] = to_bf16_grid(w) if bf16 else w
            b = _rng(seed, i, _T_BIAS).standard_normal(l["out"]) * bias_std
            p["bias"] = b.astype(np.float32)
        params.append(p)
    return params


def make_input(shape, seed, dist="normal", bf16=False):
    g = _rng(seed, -1, _T_INPUT)
    if dist == "normal":
        x = g.standard_normal(shape).astype(np.float32)
    elif dist == "uniform":
        x = g.uniform(-1.0, 1.0, shape).astype(np.float32)
    else:
        raise ValueError(dist)
    return to_bf16_grid(x) if bf16 else x


def make_labels(n, num_classes, seed):
    return _rng(seed, -1, _T_LABEL).integers(0, num_classes, n).astype(np.int32)


class Workload:
    """One benchmark/parity configuration: layer list, parameters, input."""

    def __init__(self, name, layers, in_shape, dtype, seed, dist, training=False, num_classes=None):
        self.name, self.layers, self.in_shape = name, layers, tuple(in_shape)
        self.dtype, self.seed, self.dist, self.training = dtype, seed, dist, training
        self.num_classes = num_classes
        self._params = None
        self._x = None

    @property
    def bf16(self):
        return self.dtype == "bf16"

    @property
    def params(self):
        if self._params is None:
            self._params = make_params(self.layers, self.in_shape[1], self.seed, self.bf16)
        return self._params

    @property
    def x(self):
        if self._x is None:
            self._x = make_input(self.in_shape, self.seed, self.dist, self.bf16)
        return self._x

    @property
    def labels(self):
        return make_labels(self.in_shape[0], self.num_classes, self.seed)


def config(idx: int, batch: int | None = None, hw: int | None = None, dtype: str | None = None) -> Workload:
    """The five configurations of the benchmark plus the paper's MLP workload (5), a depthwise-separable chain (6), a SqueezeNet-shaped list with channel concatenations (7) and a DenseNet-121-shaped list with pre-activation convolutions (8); ``batch`` / ``hw`` shrink a config for parity tests and ``dtype``
    overrides its storage type (same seed, same layer list)."""
    wk = _config(idx, batch, hw)
    if dtype is not None:
        wk.dtype = dtype
    return wk


def _config(idx, batch, hw):
    seed = BASE_SEED + idx
    if idx == 0:
        return Workload("single_block_fp32", single_block_layers(), (batch or 1, 3, hw or 32, hw or 32),
                        "f32", seed, "uniform")
    if idx == 1:
        return Workload("cnn5_fp32", small_cnn_layers(), (batch or 64, 3, hw or 32, hw or 32),
                        "f32", seed, "normal")
    if idx == 2:
        return Workload("resnet18_bf16", resnet18_layers(), (batch or 32, 3, hw or 224, hw or 224),
                        "bf16", seed, "normal")
    if idx == 3:
        return Workload("resnet50_bf16", resnet50_layers(), (batch or 64, 3, hw or 224, hw or 224),
                        "bf16", seed, "normal")
    if idx == 4:
        return Workload("resnet18_train_bf16", resnet18_layers(), (batch or 32, 3, hw or 224, hw or 224),
                        "bf16", seed, "normal", training=True, num_classes=1000)
    if idx == 5:   # hw = number of features here (the input is [batch, features, 1, 1])
        return Workload("mlp3_bf16", mlp_layers(hw or 8192), (batch or 64, hw or 8192, 1, 1), "bf16", seed, "normal")
    if idx == 6:
        return Workload("separable_bf16", separable_layers(), (batch or 64, 3, hw or 224, hw or 224), "bf16", seed, "normal")
    if idx == 7:
        return Workload("squeezenet_bf16", squeezenet_layers(), (batch or 64, 3, hw or 224, hw or 224), "bf16", seed, "normal")
    if idx == 8:
        return Workload("densenet121_bf16", densenet_layers(), (batch or 64, 3, hw or 224, hw or 224), "bf16", seed, "normal")
    raise ValueError(idx)
