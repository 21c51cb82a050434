"""CPU checker ("oracle") for the CNN layer-chain hot path -- TEST INFRASTRUCTURE ONLY.

A thin ctypes wrapper around ``sol_oracle.c`` (plain fp64 loop nests, one per
layer definition) plus the network-level composition of those layers.  Only
tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the product path never does, and this package imports nothing from
the product package.

All arrays are ``numpy.float64`` in logical layout: activations ``[N,C,H,W]``,
convolution weights ``[K,C,R,S]``, linear weights ``[Out,In]``.

Fused-block order (the problem statement of the library: conv, folded BN,
residual, ReLU, optional pool): ``conv -> BN -> (+ residual) -> act -> pool``.
BN is evaluated explicitly here, never folded.  In bf16 mode the result of
every layer is rounded to the nearest bf16 value at the point where the HIP
path stores it (once per fused layer, after the pool), with everything before
that kept in fp64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sol_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C checker with gcc (-O2, OpenMP on outermost loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.orc_bf16.restype = C.c_double
        _lib.orc_bf16.argtypes = [C.c_double]
        _lib.orc_softmax_ce.restype = C.c_double
        _lib.orc_out_size.restype = C.c_int
    return _lib


def threads() -> int:
    """Number of threads the OpenMP loops will use (for the CPU-baseline report)."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        return int(env.split(",")[0])
    return len(os.sched_getaffinity(0))


def _d(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _i(*v):
    return [C.c_int(int(x)) for x in v]


def out_size(n, k, s, p):
    return lib().orc_out_size(*_i(n, k, s, p))


# ------------------------------------------------------------------ forward layers
def conv2d(x, w, bias=None, stride=(1, 1), pad=(0, 0)):
    x, w = _d(x), _d(w)
    bias = _d(bias) if bias is not None else None
    N, Cc, H, W = x.shape
    K, C2, R, S = w.shape
    assert Cc == C2
    Ho, Wo = out_size(H, R, stride[0], pad[0]), out_size(W, S, stride[1], pad[1])
    y = np.empty((N, K, Ho, Wo), np.float64)
    lib().orc_conv2d(_p(x), _p(w), _p(bias), _p(y), *_i(N, Cc, H, W, K, R, S, stride[0], stride[1], pad[0], pad[1]))
    return y


def dwconv2d(x, w, bias=None, stride=(1, 1), pad=(0, 0)):
    """Depthwise convolution (groups == channels, one filter per channel); w: [C,1,R,S] or [C,R,S]."""
    x, w = _d(x), _d(w)
    bias = _d(bias) if bias is not None else None
    N, Cc, H, W = x.shape
    w = w.reshape(w.shape[0], w.shape[-2], w.shape[-1])
    C2, R, S = w.shape
    assert Cc == C2
    Ho, Wo = out_size(H, R, stride[0], pad[0]), out_size(W, S, stride[1], pad[1])
    y = np.empty((N, Cc, Ho, Wo), np.float64)
    lib().orc_dwconv2d(_p(x), _p(np.ascontiguousarray(w)), _p(bias), _p(y), *_i(N, Cc, H, W, R, S, stride[0], stride[1], pad[0], pad[1]))
    return y


def conv2d_points(x, w, bias, coords, stride=(1, 1), pad=(0, 0)):
    """Convolution outputs at the given (n,k,p,q) coordinates only."""
    x, w = _d(x), _d(w)
    bias = _d(bias) if bias is not None else None
    coords = np.ascontiguousarray(coords, dtype=np.int32)
    N, Cc, H, W = x.shape
    K, _, R, S = w.shape
    out = np.empty(len(coords), np.float64)
    lib().orc_conv2d_points(_p(x), _p(w), _p(bias), _p(coords), C.c_int(len(coords)), _p(out),
                            *_i(N, Cc, H, W, K, R, S, stride[0], stride[1], pad[0], pad[1]))
    return out


def bn_infer(x, gamma, beta, mean, var, eps=1e-5):
    x = _d(x)
    N, Cc = x.shape[:2]
    y = np.empty_like(x)
    lib().orc_bn_infer(_p(x), _p(_d(gamma)), _p(_d(beta)), _p(_d(mean)), _p(_d(var)), C.c_double(eps), _p(y),
                       *_i(N, Cc, x[0, 0].size))
    return y


def bn_infer_points(v, ch, gamma, beta, mean, var, eps=1e-5):
    v = _d(v)
    ch = np.ascontiguousarray(ch, dtype=np.int32)
    y = np.empty_like(v)
    lib().orc_bn_infer_points(_p(v), _p(ch), _p(_d(gamma)), _p(_d(beta)), _p(_d(mean)), _p(_d(var)), C.c_double(eps),
                              _p(y), C.c_int(v.size))
    return y


def bn_train(x, gamma, beta, eps=1e-5):
    x = _d(x)
    N, Cc = x.shape[:2]
    y = np.empty_like(x)
    mean, var = np.empty(Cc), np.empty(Cc)
    lib().orc_bn_train(_p(x), _p(_d(gamma)), _p(_d(beta)), C.c_double(eps), _p(y), _p(mean), _p(var),
                       *_i(N, Cc, x[0, 0].size))
    return y, mean, var


def relu(x):
    x = _d(x)
    y = np.empty_like(x)
    lib().orc_relu(_p(x), _p(y), C.c_size_t(x.size))
    return y


def add(a, b):
    a, b = _d(a), _d(b)
    assert a.shape == b.shape
    y = np.empty_like(a)
    lib().orc_add(_p(a), _p(b), _p(y), C.c_size_t(a.size))
    return y


def maxpool(x, k=(2, 2), stride=(2, 2), pad=(0, 0)):
    x = _d(x)
    N, Cc, H, W = x.shape
    Ho, Wo = out_size(H, k[0], stride[0], pad[0]), out_size(W, k[1], stride[1], pad[1])
    y = np.empty((N, Cc, Ho, Wo), np.float64)
    arg = np.empty((N, Cc, Ho, Wo), np.int32)
    lib().orc_maxpool(_p(x), _p(y), _p(arg), *_i(N, Cc, H, W, k[0], k[1], stride[0], stride[1], pad[0], pad[1]))
    return y, arg


def avgpool(x, k=(2, 2), stride=(2, 2), pad=(0, 0), count_pad=True):
    x = _d(x)
    N, Cc, H, W = x.shape
    Ho, Wo = out_size(H, k[0], stride[0], pad[0]), out_size(W, k[1], stride[1], pad[1])
    y = np.empty((N, Cc, Ho, Wo), np.float64)
    lib().orc_avgpool(_p(x), _p(y), *_i(N, Cc, H, W, k[0], k[1], stride[0], stride[1], pad[0], pad[1], count_pad))
    return y


def gap(x):
    x = _d(x)
    N, Cc = x.shape[:2]
    y = np.empty((N, Cc), np.float64)
    lib().orc_gap(_p(x), _p(y), *_i(N, Cc, x[0, 0].size))
    return y


def linear(x, w, b=None):
    x, w = _d(x), _d(w)
    b = _d(b) if b is not None else None
    M, I = x.shape
    O = w.shape[0]
    assert w.shape[1] == I
    y = np.empty((M, O), np.float64)
    lib().orc_linear(_p(x), _p(w), _p(b), _p(y), *_i(M, I, O))
    return y


def bf16(v: float) -> float:
    return lib().orc_bf16(float(v))


def round_bf16(x):
    y = _d(x).copy()
    lib().orc_round_bf16(_p(y), C.c_size_t(y.size))
    return y


def pool(x, pd):
    """Apply a pool-dict; returns (y, argmax or None)."""
    k, s, p = (pd["kh"], pd["kw"]), (pd["sh"], pd["sw"]), (pd["ph"], pd["pw"])
    if pd["kind"] == "max":
        return maxpool(x, k, s, p)
    if pd["kind"] == "avg":
        return avgpool(x, k, s, p, bool(pd.get("count_pad", 1))), None
    raise ValueError(pd["kind"])


def concat(a, b):
    """Channel concatenation of two NCHW tensors of equal n, h, w: out[:, :Ca] = a, out[:, Ca:] = b (the join of
    parallel branches in the SqueezeNet / DenseNet-shaped networks of the paper's evaluation, Sec. VI)."""
    a, b = _d(a), _d(b)
    if a.shape[0] != b.shape[0] or a.shape[2:] != b.shape[2:]:
        raise ValueError(f"concat: {a.shape} vs {b.shape}")
    out = np.empty((a.shape[0], a.shape[1] + b.shape[1]) + a.shape[2:], np.float64)
    for n in range(a.shape[0]):
        for c in range(a.shape[1]):
            out[n, c] = a[n, c]
        for c in range(b.shape[1]):
            out[n, a.shape[1] + c] = b[n, c]
    return out


# ----------------------------------------------------------------- backward layers
def conv2d_dgrad(dy, w, x_shape, stride=(1, 1), pad=(0, 0)):
    dy, w = _d(dy), _d(w)
    N, Cc, H, W = x_shape
    K, _, R, S = w.shape
    dx = np.empty(x_shape, np.float64)
    lib().orc_conv2d_dgrad(_p(dy), _p(w), _p(dx), *_i(N, Cc, H, W, K, R, S, stride[0], stride[1], pad[0], pad[1]))
    return dx


def conv2d_wgrad(x, dy, w_shape, stride=(1, 1), pad=(0, 0)):
    x, dy = _d(x), _d(dy)
    N, Cc, H, W = x.shape
    K, _, R, S = w_shape
    dw, db = np.empty(w_shape, np.float64), np.empty(K, np.float64)
    lib().orc_conv2d_wgrad(_p(x), _p(dy), _p(dw), _p(db), *_i(N, Cc, H, W, K, R, S, stride[0], stride[1], pad[0], pad[1]))
    return dw, db


def bn_train_bwd(x, dy, gamma, mean, var, eps=1e-5):
    x, dy = _d(x), _d(dy)
    N, Cc = x.shape[:2]
    dx, dg, db = np.empty_like(x), np.empty(Cc), np.empty(Cc)
    lib().orc_bn_train_bwd(_p(x), _p(dy), _p(_d(gamma)), _p(_d(mean)), _p(_d(var)), C.c_double(eps),
                           _p(dx), _p(dg), _p(db), *_i(N, Cc, x[0, 0].size))
    return dx, dg, db


def relu_bwd(y, dy):
    y, dy = _d(y), _d(dy)
    dx = np.empty_like(y)
    lib().orc_relu_bwd(_p(y), _p(dy), _p(dx), C.c_size_t(y.size))
    return dx


def maxpool_bwd(dy, argmax, x_shape):
    dy = _d(dy)
    argmax = np.ascontiguousarray(argmax, dtype=np.int32)
    N, Cc, H, W = x_shape
    dx = np.empty(x_shape, np.float64)
    lib().orc_maxpool_bwd(_p(dy), _p(argmax), _p(dx), *_i(N, Cc, H, W, dy.shape[2], dy.shape[3]))
    return dx


def avgpool_bwd(dy, x_shape, k, stride, pad, count_pad=True):
    dy = _d(dy)
    N, Cc, H, W = x_shape
    dx = np.empty(x_shape, np.float64)
    lib().orc_avgpool_bwd(_p(dy), _p(dx), *_i(N, Cc, H, W, k[0], k[1], stride[0], stride[1], pad[0], pad[1], count_pad))
    return dx


def gap_bwd(dy, x_shape):
    dy = _d(dy)
    N, Cc, H, W = x_shape
    dx = np.empty(x_shape, np.float64)
    lib().orc_gap_bwd(_p(dy), _p(dx), *_i(N, Cc, H * W))
    return dx


def linear_bwd(x, w, dy):
    x, w, dy = _d(x), _d(w), _d(dy)
    M, I = x.shape
    O = w.shape[0]
    dx, dw, db = np.empty((M, I)), np.empty((O, I)), np.empty(O)
    lib().orc_linear_bwd(_p(x), _p(w), _p(dy), _p(dx), _p(dw), _p(db), *_i(M, I, O))
    return dx, dw, db


def softmax_ce(z, labels, want_grad=True):
    z = _d(z)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    N, K = z.shape
    dz = np.empty_like(z) if want_grad else None
    loss = lib().orc_softmax_ce(_p(z), _p(labels), _p(dz), *_i(N, K))
    return loss, dz


def sgd(w, v, g, lr, mu):
    """In-place momentum SGD on fp64 arrays: v <- mu v + g ; w <- w - lr v."""
    assert w.dtype == np.float64 and v.dtype == np.float64 and w.flags.c_contiguous and v.flags.c_contiguous
    g = _d(g)
    lib().orc_sgd(_p(w), _p(v), _p(g), C.c_double(lr), C.c_double(mu), C.c_size_t(w.size))


# ---------------------------------------------------------------- fused layer, network
def _src_of(i, l, outs, x):
    s = l.get("src", -1)
    if s == -1:
        return x if i == 0 else outs[i - 1]
    return outs[s]


def pre_activation(x, p, bf16=False):
    """BN + ReLU on the INPUT side of a convolution (the pre-activation order of the DenseNet-shaped networks of the
    paper's evaluation, Sec. VI): relu(pre_gamma (x - pre_mean) / sqrt(pre_var + eps) + pre_beta), per input channel.
    In bf16 mode the activated tensor is a rounding point, exactly as if a stand-alone BN-ReLU layer had stored it:
    the HIP path feeds it to the matrix cores in bf16.  Zero padding of the convolution applies to this tensor."""
    y = relu(bn_infer(x, p["pre_gamma"], p["pre_beta"], p["pre_mean"], p["pre_var"], p.get("eps", 1e-5)))
    return round_bf16(y) if bf16 else y


def fused_conv(x, p, l, residual=None, bf16=False, want_prepool=False):
    """[BN -> ReLU on the input ->] conv -> explicit BN -> (+residual) -> act -> pool -> (bf16 store).
    Returns (y, argmax, prepool)."""
    cv = dwconv2d if l.get("dw") else conv2d
    if l.get("pre_bn"):
        x = pre_activation(x, p, bf16)
    y = cv(x, p["w"], p.get("bias"), (l["sh"], l["sw"]), (l["ph"], l["pw"]))
    if l["bn"]:
        y = bn_infer(y, p["gamma"], p["beta"], p["mean"], p["var"], p.get("eps", 1e-5))
    if residual is not None:
        y = add(y, residual)
    if l["act"] == "relu":
        y = relu(y)
    arg, pre = None, (y if want_prepool else None)
    if l.get("pool"):
        y, arg = pool(y, l["pool"])
    if bf16:
        y = round_bf16(y)
    return y, arg, pre


def fused_conv_points(x, p, l, coords, residual=None, bf16=False):
    """The fused block (without pool) evaluated at output coordinates (n,k,p,q) only."""
    coords = np.ascontiguousarray(coords, dtype=np.int32)
    y = conv2d_points(x, p["w"], p.get("bias"), coords, (l["sh"], l["sw"]), (l["ph"], l["pw"]))
    if l["bn"]:
        y = bn_infer_points(y, coords[:, 1], p["gamma"], p["beta"], p["mean"], p["var"], p.get("eps", 1e-5))
    if residual is not None:
        y = add(y, _d(residual)[coords[:, 0], coords[:, 1], coords[:, 2], coords[:, 3]])
    if l["act"] == "relu":
        y = relu(y)
    if bf16:
        y = round_bf16(y)
    return y


def network_forward(layers, params, x, bf16=False, return_all=False):
    """Inference forward of a layer list; the output of every layer is a storage point."""
    x = _d(x)
    outs, args = [], []
    for i, l in enumerate(layers):
        src = _src_of(i, l, outs, x)
        arg = None
        if l["kind"] == "conv":
            res = outs[l["res"]] if l.get("res", -1) >= 0 else None
            y, arg, _ = fused_conv(src, params[i], l, res, bf16)
        elif l["kind"] == "pool":
            y, arg = pool(src, l["pool"])
            if bf16:
                y = round_bf16(y)
        elif l["kind"] == "gap":
            y = gap(src)
            if bf16:
                y = round_bf16(y)
        elif l["kind"] == "concat":
            y = concat(src, outs[l["res"]])             # stored values only move: nothing to round
        elif l["kind"] == "linear":
            y = linear(src.reshape(src.shape[0], -1), params[i]["w"], params[i].get("bias"))
            if l.get("act") == "relu":
                y = relu(y)
            if bf16:
                y = round_bf16(y)
        else:
            raise ValueError(l["kind"])
        outs.append(y)
        args.append(arg)
    return (outs, args) if return_all else outs[-1]


# ------------------------------------------------------------------------ training step
def _rnd(a, bf16):
    return round_bf16(a) if bf16 else a


def network_train_step(layers, params, x, labels, lr, mu, velocity=None, bf16=False, eps=1e-5, forced=None):
    """One training step of a layer list: forward with batch-statistics BN, softmax cross-entropy
    (batch mean), full backward, SGD with momentum (v <- mu v + g ; w <- w - lr v).

    Rounding points in bf16 mode (where the HIP path stores a tensor): the convolution output z that
    the batch statistics are taken from, every layer output, every accumulated activation gradient
    (a tensor with several consumers receives its contributions in descending consumer order, each
    added to the stored value and stored again), dz of every BN; statistics, weight gradients,
    master weights and velocities stay unrounded.  Fused pools are not part of the training path.

    forced = {"outs": [...], "z": [...]} (entries may be None) replaces the stored forward tensors by the
    given ones, layer by layer, before anything else reads them: the backward pass, which is linear in the
    incoming gradient once the stored tensors are fixed, can then be compared on its own.

    Returns a dict: loss, outs, grads (per layer: w, bias, gamma, beta), new_params, velocity,
    stats (per layer: mean, var), dacts (stored gradient of every layer output).
    """
    x = _d(x)
    n_layers = len(layers)
    outs, saved = [], []
    for i, l in enumerate(layers):
        src = _src_of(i, l, outs, x)
        sv = {}
        if l["kind"] == "conv":
            assert not l.get("pool"), "fused pool is not supported in training"
            p = params[i]
            z = conv2d(src, p["w"], p.get("bias"), (l["sh"], l["sw"]), (l["ph"], l["pw"]))
            if l["bn"]:
                z = _rnd(z, bf16)
                if forced is not None and forced["z"][i] is not None:
                    z = _d(forced["z"][i]).reshape(z.shape)
                y, mean, var = bn_train(z, p["gamma"], p["beta"], eps)
                sv.update(z=z, mean=mean, var=var)
            else:
                y = z
            if l.get("res", -1) >= 0:
                y = add(y, outs[l["res"]])
            if l["act"] == "relu":
                y = relu(y)
            y = _rnd(y, bf16)
        elif l["kind"] == "pool":
            y, arg = pool(src, l["pool"])
            sv.update(arg=arg)
            y = _rnd(y, bf16)
        elif l["kind"] == "gap":
            y = _rnd(gap(src), bf16)
        elif l["kind"] == "linear":
            y = linear(src.reshape(src.shape[0], -1), params[i]["w"], params[i].get("bias"))
            if l.get("act") == "relu":
                y = relu(y)
            y = _rnd(y, bf16)
        else:
            raise ValueError(l["kind"])
        if forced is not None and forced["outs"][i] is not None:
            y = _d(forced["outs"][i]).reshape(y.shape)
        outs.append(y)
        saved.append(sv)

    loss, dlogits = softmax_ce(outs[-1].reshape(outs[-1].shape[0], -1), labels)
    dacts = [None] * n_layers
    dacts[-1] = _rnd(dlogits.reshape(outs[-1].shape), bf16)

    def contribute(t, c):
        if t < 0:
            return                      # gradient w.r.t. the network input is not needed
        dacts[t] = _rnd(c, bf16) if dacts[t] is None else _rnd(add(dacts[t], c), bf16)

    grads = [dict() for _ in layers]
    for i in range(n_layers - 1, -1, -1):
        l, p, sv = layers[i], params[i], saved[i]
        s = l.get("src", -1)
        t = (i - 1) if s == -1 else s
        src = x if t < 0 else outs[t]
        dy = dacts[i]
        if dy is None:
            continue
        if l["kind"] == "linear":
            g = relu_bwd(outs[i], dy) if l.get("act") == "relu" else dy
            xin = src.reshape(src.shape[0], -1)
            dx, dw, db = linear_bwd(xin, p["w"], g)
            grads[i].update(w=dw, bias=db)
            contribute(t, dx.reshape(src.shape))
        elif l["kind"] == "gap":
            contribute(t, gap_bwd(dy.reshape(dy.shape[0], dy.shape[1]), src.shape))
        elif l["kind"] == "pool":
            pd = l["pool"]
            if pd["kind"] == "max":
                contribute(t, maxpool_bwd(dy, sv["arg"], src.shape))
            else:
                contribute(t, avgpool_bwd(dy, src.shape, (pd["kh"], pd["kw"]), (pd["sh"], pd["sw"]),
                                          (pd["ph"], pd["pw"]), bool(pd.get("count_pad", 1))))
        elif l["kind"] == "conv":
            g = relu_bwd(outs[i], dy) if l["act"] == "relu" else dy
            if l.get("res", -1) >= 0:
                contribute(l["res"], g)
            if l["bn"]:
                dz, dg, dbt = bn_train_bwd(sv["z"], g, p["gamma"], sv["mean"], sv["var"], eps)
                grads[i].update(gamma=dg, beta=dbt)
                dz = _rnd(dz, bf16)
            else:
                dz = g
            dw, db = conv2d_wgrad(src, dz, p["w"].shape, (l["sh"], l["sw"]), (l["ph"], l["pw"]))
            grads[i].update(w=dw)
            if not l["bn"]:
                grads[i].update(bias=db)
            if t >= 0:
                contribute(t, conv2d_dgrad(dz, p["w"], src.shape, (l["sh"], l["sw"]), (l["ph"], l["pw"])))

    velocity = velocity if velocity is not None else [dict() for _ in layers]
    new_params = []
    for i, (p, g) in enumerate(zip(params, grads)):
        q = dict(p)
        for k, gk in g.items():
            w = _d(p[k]).copy()
            v = _d(velocity[i][k]).copy() if k in velocity[i] else np.zeros_like(w)
            sgd(w, v, gk, lr, mu)
            q[k] = w
            velocity[i][k] = v
        new_params.append(q)
    return {"loss": loss, "outs": outs, "grads": grads, "new_params": new_params, "velocity": velocity,
            "stats": [{k: sv[k] for k in ("mean", "var") if k in sv} for sv in saved], "dacts": dacts}
