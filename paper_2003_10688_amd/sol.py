"""Thin Python binding of libsol_mi355.so (see include/sol.h): same names, argument marshalling only.

PyTorch is used for device memory and streams; every step of the computation runs inside the HIP
library.  There is no CPU fallback: if the library is missing or there is no GPU, calls raise.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SOL_MI355_LIB") or os.path.join(_HERE, "libsol_mi355.so")

F32, BF16 = 0, 1
ACT_NONE, ACT_RELU = 0, 1
POOL_NONE, POOL_MAX, POOL_AVG = 0, 1, 2
LAYER_CONV, LAYER_POOL, LAYER_GAP, LAYER_LINEAR, LAYER_DWCONV, LAYER_CONCAT = 0, 1, 2, 3, 4, 5
NET_TRAINING, NET_KEEP_ACTIVATIONS = 1, 2
NT_W, NT_GAMMA, NT_BETA, NT_BIAS, NT_GRAD_W, NT_GRAD_GAMMA, NT_GRAD_BETA, NT_GRAD_BIAS, NT_MEAN, NT_VAR = range(10)
NT_VEL_W, NT_VEL_GAMMA, NT_VEL_BETA, NT_VEL_BIAS = range(10, 14)

STATUS = {0: "SOL_OK", 1: "SOL_ERR_NULL", 2: "SOL_ERR_SHAPE", 3: "SOL_ERR_DTYPE", 4: "SOL_ERR_ALIGN",
          5: "SOL_ERR_WORKSPACE", 6: "SOL_ERR_UNSUPPORTED", 7: "SOL_ERR_HIP"}


class PoolDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("kind", "kh", "kw", "sh", "sw", "ph", "pw", "count_pad")]


class TensorDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("n", "h", "w", "c", "dtype")]


class ConvDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("cout", "cin", "kh", "kw", "sh", "sw", "ph", "pw")]


class Layer(C.Structure):
    _fields_ = [("kind", C.c_int), ("conv", ConvDesc), ("has_bn", C.c_int), ("act", C.c_int),
                ("pool", PoolDesc), ("out_features", C.c_int), ("src", C.c_int), ("res", C.c_int), ("pre_bn", C.c_int)]


class SolError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"{STATUS.get(status, status)}: {text}")
        self.status = status


_lib = None


def lib():
    """Loads the HIP library; fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(LIB_PATH)
        L.sol_last_error.restype = C.c_char_p
        L.sol_version.restype = C.c_char_p
        L.sol_packed_weight_bytes.restype = C.c_size_t
        L.sol_packed_weight_bytes.argtypes = [C.POINTER(ConvDesc), C.c_int]
        L.sol_packed_dw_weight_bytes.restype = C.c_size_t
        L.sol_packed_dw_weight_bytes.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int]
        L.sol_network_param_bytes.restype = C.c_size_t
        L.sol_network_param_bytes.argtypes = [C.c_void_p]
        L.sol_network_workspace_bytes.restype = C.c_size_t
        L.sol_network_workspace_bytes.argtypes = [C.c_void_p]
        L.sol_network_num_layers.argtypes = [C.c_void_p]
        L.sol_network_destroy.argtypes = [C.c_void_p]
        L.sol_network_destroy.restype = None
        L.sol_graph_destroy.argtypes = [C.c_void_p]
        L.sol_graph_destroy.restype = None
        L.sol_graph_launch.argtypes = [C.c_void_p, C.c_void_p]
        L.sol_debug_set_conv_tile.restype = None
        L.sol_debug_probe_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.sol_debug_probe_mfma.argtypes = [C.c_int, C.c_int, C.c_void_p, C.POINTER(C.c_double), C.c_void_p]
        L.sol_network_forward_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _check(status):
    if status != 0:
        raise SolError(status, lib().sol_last_error().decode())


def _ptr(t):
    if t is None:
        return C.c_void_p(0)
    if isinstance(t, torch.Tensor):
        assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous GPU tensors"
        return C.c_void_p(t.data_ptr())
    return C.c_void_p(int(t))


def _stream(stream=None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def torch_dtype(dt):
    return torch.bfloat16 if dt == BF16 else torch.float32


def dtype_of(t):
    return BF16 if t.dtype == torch.bfloat16 else F32


# ---- layout marshalling (logical NCHW numpy  <->  NHWC device tensors) --------------------------------
def to_device_nhwc(a, dt, device="cuda:0"):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if t.dim() == 4:
        t = t.permute(0, 2, 3, 1)
    return t.contiguous().to(device=device, dtype=torch_dtype(dt))


def to_host_nchw(t):
    t = t.detach().to("cpu")
    if t.dtype == torch.bfloat16:
        t = t.to(torch.float32)
    if t.dim() == 4:
        t = t.permute(0, 3, 1, 2)
    return t.contiguous().numpy()


def dev_f32(a, device="cuda:0"):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


def pool_desc(pd):
    if pd is None:
        return None
    kind = {"max": POOL_MAX, "avg": POOL_AVG, "none": POOL_NONE}[pd["kind"]] if isinstance(pd["kind"], str) else pd["kind"]
    return PoolDesc(kind, pd["kh"], pd["kw"], pd["sh"], pd["sw"], pd["ph"], pd["pw"], int(pd.get("count_pad", 1)))


def tensor_desc(t):
    n, h, w, c = t.shape
    return TensorDesc(n, h, w, c, dtype_of(t))


# ---- single-layer entry points ------------------------------------------------------------------------
def sol_out_size(n, k, s, p):
    return lib().sol_out_size(C.c_int(n), C.c_int(k), C.c_int(s), C.c_int(p))


def sol_packed_weight_bytes(cd, dt):
    return lib().sol_packed_weight_bytes(C.byref(cd), C.c_int(dt))


def sol_pack_conv_weights(cd, dt, w_oihw, stream=None):
    """w_oihw: device fp32 [cout][cin][kh][kw] -> packed device buffer (uint8 tensor)."""
    packed = torch.empty(sol_packed_weight_bytes(cd, dt), dtype=torch.uint8, device=w_oihw.device)
    _check(lib().sol_pack_conv_weights(C.byref(cd), C.c_int(dt), _ptr(w_oihw), _ptr(packed), _stream(stream)))
    return packed


def sol_unpack_conv_weights(cd, dt, packed, stream=None):
    w = torch.empty((cd.cout, cd.cin, cd.kh, cd.kw), dtype=torch.float32, device=packed.device)
    _check(lib().sol_unpack_conv_weights(C.byref(cd), C.c_int(dt), _ptr(packed), _ptr(w), _stream(stream)))
    return w


def sol_fold_bn(c, gamma, beta, mean, var, bias, eps, device="cuda:0", stream=None):
    scale = torch.empty(c, dtype=torch.float32, device=device)
    shift = torch.empty(c, dtype=torch.float32, device=device)
    _check(lib().sol_fold_bn(C.c_int(c), _ptr(gamma), _ptr(beta), _ptr(mean), _ptr(var), _ptr(bias),
                             C.c_float(eps), _ptr(scale), _ptr(shift), _stream(stream)))
    return scale, shift


def sol_conv2d_fused(x, cd, w_packed, scale=None, shift=None, residual=None, act=ACT_NONE, pool=None,
                     want_argmax=False, want_prepool=False, stream=None):
    """x: NHWC device tensor.  Returns (y, argmax or None, prepool or None)."""
    n, h, w, _ = x.shape
    ho, wo = sol_out_size(h, cd.kh, cd.sh, cd.ph), sol_out_size(w, cd.kw, cd.sw, cd.pw)
    hy, wy = ho, wo
    pd = pool if isinstance(pool, PoolDesc) or pool is None else pool_desc(pool)
    if pd is not None and pd.kind != POOL_NONE:
        hy, wy = sol_out_size(ho, pd.kh, pd.sh, pd.ph), sol_out_size(wo, pd.kw, pd.sw, pd.pw)
    y = torch.empty((n, max(hy, 0), max(wy, 0), cd.cout), dtype=x.dtype, device=x.device)
    arg = torch.empty(y.shape, dtype=torch.int32, device=x.device) if want_argmax else None
    pre = torch.empty((n, max(ho, 0), max(wo, 0), cd.cout), dtype=x.dtype, device=x.device) if want_prepool else None
    xd = tensor_desc(x)
    _check(lib().sol_conv2d_fused(C.byref(xd), _ptr(x), C.byref(cd), _ptr(w_packed), _ptr(scale), _ptr(shift),
                                  _ptr(residual), C.c_int(act), C.byref(pd) if pd is not None else None,
                                  _ptr(y), _ptr(arg), _ptr(pre), _stream(stream)))
    return y, arg, pre


def sol_conv2d_preact_fused(x, cd, w_packed, pre_scale=None, pre_shift=None, scale=None, shift=None, residual=None, act=ACT_NONE,
                            pool=None, channels=None, stream=None):
    """x: NHWC device tensor; channels: read only the first `channels` channels of every pixel of x (a channel prefix of
    a wider tensor; default: all).  Returns y."""
    n, h, w, ctot = x.shape
    c = channels or ctot
    ho, wo = sol_out_size(h, cd.kh, cd.sh, cd.ph), sol_out_size(w, cd.kw, cd.sw, cd.pw)
    pd = pool if isinstance(pool, PoolDesc) or pool is None else pool_desc(pool)
    if pd is not None and pd.kind != POOL_NONE:
        ho, wo = sol_out_size(ho, pd.kh, pd.sh, pd.ph), sol_out_size(wo, pd.kw, pd.sw, pd.pw)
    y = torch.empty((n, max(ho, 0), max(wo, 0), cd.cout), dtype=x.dtype, device=x.device)
    xd = TensorDesc(n, h, w, c, dtype_of(x))
    _check(lib().sol_conv2d_preact_fused(C.byref(xd), _ptr(x), C.c_int(ctot if c != ctot else 0), _ptr(pre_scale), _ptr(pre_shift),
                                         C.byref(cd), _ptr(w_packed), _ptr(scale), _ptr(shift), _ptr(residual), C.c_int(act),
                                         C.byref(pd) if pd is not None else None, _ptr(y), _stream(stream)))
    return y


def sol_bottleneck_fused(x, mid, w1, s1, h1, w2, s2, h2, w3, s3, h3, stream=None):
    """x: NHWC bf16 device tensor; w*: packed weights; s*/h*: folded scale / shift.  Returns y (same shape as x)."""
    y = torch.empty_like(x)
    xd = tensor_desc(x)
    _check(lib().sol_bottleneck_fused(C.byref(xd), _ptr(x), C.c_int(mid), _ptr(w1), _ptr(s1), _ptr(h1), _ptr(w2), _ptr(s2), _ptr(h2),
                                      _ptr(w3), _ptr(s3), _ptr(h3), _ptr(y), _stream(stream)))
    return y


def sol_expand_reduce_fused(t, c4, w3, s3, h3, shortcut, cz, w1, s1, h1, stream=None):
    """t: NHWC bf16 device tensor [n,h,w,256]; shortcut: [n,h,w,c4]; w*: packed weights; s*/h*: folded scale / shift.
    Returns (y [n,h,w,c4], z [n,h,w,cz])."""
    n, h, w, _ = t.shape
    y = torch.empty((n, h, w, c4), dtype=t.dtype, device=t.device)
    z = torch.empty((n, h, w, cz), dtype=t.dtype, device=t.device)
    td = tensor_desc(t)
    _check(lib().sol_expand_reduce_fused(C.byref(td), _ptr(t), C.c_int(c4), _ptr(w3), _ptr(s3), _ptr(h3), _ptr(shortcut), _ptr(y),
                                         C.c_int(cz), _ptr(w1), _ptr(s1), _ptr(h1), _ptr(z), _stream(stream)))
    return y, z


def sol_pack_dwconv_weights(c, kh, kw, dt, w_c1hw, stream=None):
    """w_c1hw: device fp32 [c][1][kh][kw] -> packed device buffer (uint8 tensor)."""
    packed = torch.empty(lib().sol_packed_dw_weight_bytes(c, kh, kw, dt), dtype=torch.uint8, device=w_c1hw.device)
    _check(lib().sol_pack_dwconv_weights(C.c_int(c), C.c_int(kh), C.c_int(kw), C.c_int(dt), _ptr(w_c1hw), _ptr(packed),
                                         _stream(stream)))
    return packed


def sol_dwconv2d_fused(x, cd, w_packed, scale=None, shift=None, residual=None, act=ACT_NONE, stream=None):
    """x: NHWC device tensor; cd.cin == cd.cout == channels.  Returns y."""
    n, h, w, c = x.shape
    ho, wo = sol_out_size(h, cd.kh, cd.sh, cd.ph), sol_out_size(w, cd.kw, cd.sw, cd.pw)
    y = torch.empty((n, max(ho, 0), max(wo, 0), c), dtype=x.dtype, device=x.device)
    xd = tensor_desc(x)
    _check(lib().sol_dwconv2d_fused(C.byref(xd), _ptr(x), C.byref(cd), _ptr(w_packed), _ptr(scale), _ptr(shift),
                                    _ptr(residual), C.c_int(act), _ptr(y), _stream(stream)))
    return y


def sol_linear(x, w_packed, bias, out_f, act=ACT_NONE, stream=None):
    m, in_f = x.shape
    y = torch.empty((m, out_f), dtype=x.dtype, device=x.device)
    _check(lib().sol_linear(C.c_int(m), C.c_int(in_f), C.c_int(out_f), C.c_int(dtype_of(x)), _ptr(x), _ptr(w_packed),
                            _ptr(bias), C.c_int(act), _ptr(y), _stream(stream)))
    return y


def sol_pool(x, pd, want_argmax=False, stream=None):
    pd = pd if isinstance(pd, PoolDesc) else pool_desc(pd)
    n, h, w, c = x.shape
    ho, wo = sol_out_size(h, pd.kh, pd.sh, pd.ph), sol_out_size(w, pd.kw, pd.sw, pd.pw)
    y = torch.empty((n, max(ho, 0), max(wo, 0), c), dtype=x.dtype, device=x.device)
    arg = torch.empty(y.shape, dtype=torch.int32, device=x.device) if want_argmax else None
    xd = tensor_desc(x)
    _check(lib().sol_pool(C.byref(xd), _ptr(x), C.byref(pd), _ptr(y), _ptr(arg), _stream(stream)))
    return y, arg


def sol_global_avgpool(x, stream=None):
    n, h, w, c = x.shape
    y = torch.empty((n, 1, 1, c), dtype=x.dtype, device=x.device)
    xd = tensor_desc(x)
    _check(lib().sol_global_avgpool(C.byref(xd), _ptr(x), _ptr(y), _stream(stream)))
    return y


def sol_debug_set_conv_tile(tile):
    lib().sol_debug_set_conv_tile(C.c_int(tile))


def sol_debug_probe_copy(dst, src, stream=None):
    """Plain device-to-device copy of src into dst (uint8 tensors of equal size, a multiple of 16 bytes)."""
    assert dst.numel() * dst.element_size() == src.numel() * src.element_size()
    _check(lib().sol_debug_probe_copy(_ptr(dst), _ptr(src), C.c_size_t(src.numel() * src.element_size()), _stream(stream)))


def sol_debug_probe_mfma(iters, workgroups, sink, stream=None):
    """Register-resident bf16 MFMA loop; returns the floating-point operations of the launch."""
    flop = C.c_double(0.0)
    _check(lib().sol_debug_probe_mfma(C.c_int(iters), C.c_int(workgroups), _ptr(sink), C.byref(flop), _stream(stream)))
    return flop.value


# ---- networks -----------------------------------------------------------------------------------------
def make_layer_array(layers):
    arr = (Layer * len(layers))()
    for i, l in enumerate(layers):
        a = arr[i]
        a.src, a.res = l.get("src", -1), l.get("res", -1)
        a.act = ACT_RELU if l.get("act") == "relu" else ACT_NONE
        a.pool = PoolDesc(POOL_NONE, 0, 0, 0, 0, 0, 0, 0)
        if l["kind"] == "conv":
            a.kind = LAYER_DWCONV if l.get("dw") else LAYER_CONV
            a.conv = ConvDesc(l["cout"], 0, l["kh"], l["kw"], l["sh"], l["sw"], l["ph"], l["pw"])
            a.has_bn = int(l["bn"])
            a.pre_bn = int(bool(l.get("pre_bn")))
            if l.get("pool"):
                a.pool = pool_desc(l["pool"])
        elif l["kind"] == "pool":
            a.kind = LAYER_POOL
            a.pool = pool_desc(l["pool"])
        elif l["kind"] == "gap":
            a.kind = LAYER_GAP
        elif l["kind"] == "concat":
            a.kind = LAYER_CONCAT
        elif l["kind"] == "linear":
            a.kind = LAYER_LINEAR
            a.out_features = l["out"]
        else:
            raise ValueError(l["kind"])
    return arr


class Network:
    """sol_network_* wrapper: plan once (create + parameter packing), then forward many times."""

    def __init__(self, layers, in_shape_nchw, dt, device="cuda:0", flags=0):
        self.layers, self.dt, self.device = layers, dt, device
        self.training = bool(flags & NET_TRAINING)
        n, c, h, w = in_shape_nchw
        self.in_desc = TensorDesc(n, h, w, c, dt)
        self._h = C.c_void_p(0)
        arr = make_layer_array(layers)
        _check(lib().sol_network_create(arr, C.c_int(len(layers)), C.byref(self.in_desc), C.c_int(flags), C.byref(self._h)))
        self.param_buf = torch.empty(max(lib().sol_network_param_bytes(self._h), 16), dtype=torch.uint8, device=device)
        self.workspace = torch.empty(max(lib().sol_network_workspace_bytes(self._h), 16), dtype=torch.uint8, device=device)
        _check(lib().sol_network_bind_params(self._h, _ptr(self.param_buf), C.c_size_t(self.param_buf.numel())))
        od = self.output_desc(-1)
        self.y = torch.empty((od.n, od.h, od.w, od.c), dtype=torch_dtype(dt), device=device)

    def output_desc(self, layer=-1):
        d = TensorDesc()
        _check(lib().sol_network_output_desc(self._h, C.c_int(layer), C.byref(d)))
        return d

    def set_params(self, params, stream=None):
        """params: per-layer dicts of numpy fp32 arrays in framework layout (w OIHW, depthwise [c][1][kh][kw], linear [out][in])."""
        for i, (l, p) in enumerate(zip(self.layers, params)):
            if l["kind"] not in ("conv", "linear"):
                continue
            w = dev_f32(p["w"], self.device)
            bn = l["kind"] == "conv" and l["bn"]
            keys = ("gamma", "beta") if self.training else ("gamma", "beta", "mean", "var")
            g, b, m, v = ([dev_f32(p[k], self.device) for k in keys] + [None, None])[:4] if bn else (None,) * 4
            bias = dev_f32(p.get("bias"), self.device)
            _check(lib().sol_network_set_params(self._h, C.c_int(i), _ptr(w), _ptr(g), _ptr(b), _ptr(m), _ptr(v),
                                                _ptr(bias), C.c_float(p.get("eps", 1e-5)), _stream(stream)))
            if l["kind"] == "conv" and l.get("pre_bn"):
                pg, pb, pm, pv = (dev_f32(p[k], self.device) for k in ("pre_gamma", "pre_beta", "pre_mean", "pre_var"))
                _check(lib().sol_network_set_pre_bn(self._h, C.c_int(i), _ptr(pg), _ptr(pb), _ptr(pm), _ptr(pv),
                                                    C.c_float(p.get("eps", 1e-5)), _stream(stream)))
        torch.cuda.synchronize()

    def forward(self, x, stream=None):
        """x: NHWC device tensor; returns the (reused) output tensor of the last layer."""
        _check(lib().sol_network_forward(self._h, _ptr(x), _ptr(self.y), _ptr(self.workspace),
                                         C.c_size_t(self.workspace.numel()), _stream(stream)))
        return self.y

    def forward_static(self, x, stream=None):
        """sol_network_forward_static: the same pass with the library's static device array as workspace."""
        _check(lib().sol_network_forward_static(self._h, _ptr(x), _ptr(self.y), _stream(stream)))
        return self.y

    def autotune(self, x, reps=10, stream=None):
        """Plan-time per-layer kernel/tile selection by timing (synchronous); returns {layer: tile id} of the changed layers."""
        _check(lib().sol_network_autotune(self._h, _ptr(x), _ptr(self.y), _ptr(self.workspace),
                                          C.c_size_t(self.workspace.numel()), C.c_int(reps), _stream(stream)))
        out = {}
        for i in range(len(self.layers)):
            t = C.c_int(0)
            _check(lib().sol_network_layer_tile(self._h, C.c_int(i), C.byref(t)))
            if t.value:
                out[i] = t.value
            b = self.block_state(i)
            if b >= 0:
                out[f"{i}b"] = b          # bottleneck ending in layer i: 1 = one depth-first launch, 0 = layer by layer
            b = self.xr_state(i)
            if b >= 0:
                out[f"{i}x"] = b          # expand-reduce pair starting in layer i: 1 = one launch, 0 = two
        return out

    def set_tiles(self, tiles):
        """Restores per-layer kernel/tile ids from an earlier autotune() of the same network ({layer: tile id})."""
        for i in range(len(self.layers)):
            _check(lib().sol_network_set_layer_tile(self._h, C.c_int(i), C.c_int(int(tiles.get(i, tiles.get(str(i), 0))))))
            if f"{i}b" in tiles:
                self.set_block(i, tiles[f"{i}b"])
            if f"{i}x" in tiles:
                self.set_xr(i, tiles[f"{i}x"])

    def graph(self, x, stream):
        """Records one forward pass on `stream` (a torch.cuda.Stream other than the default one) as a HIP graph;
        returns a callable that enqueues one replay on that stream and returns the output tensor."""
        g = C.c_void_p(0)
        _check(lib().sol_network_graph_create(self._h, _ptr(x), _ptr(self.y), _ptr(self.workspace),
                                              C.c_size_t(self.workspace.numel()), _stream(stream), C.byref(g)))
        self._graphs = getattr(self, "_graphs", []) + [g]
        self._graph_keep = getattr(self, "_graph_keep", []) + [x]

        def launch():
            _check(lib().sol_graph_launch(g, _stream(stream)))
            return self.y
        return launch

    def block_state(self, layer):
        """-1: `layer` ends no bottleneck the depth-first kernel can run; 0: runs layer by layer; 1: as one launch."""
        t = C.c_int(0)
        _check(lib().sol_network_layer_block(self._h, C.c_int(layer), C.byref(t)))
        return t.value

    def set_block(self, layer, fused):
        """Runs the bottleneck that ends in convolution `layer` as one depth-first launch (fused) or layer by layer."""
        _check(lib().sol_network_set_layer_block(self._h, C.c_int(layer), C.c_int(int(bool(fused)))))

    def xr_state(self, layer):
        """-1: `layer` starts no expand-reduce pair the depth-first kernel can run; 0: the two layers run one by one; 1: as one launch."""
        t = C.c_int(0)
        _check(lib().sol_network_layer_xr(self._h, C.c_int(layer), C.byref(t)))
        return t.value

    def set_xr(self, layer, fused):
        """Runs convolution `layer` and the 1x1 convolution behind it as one depth-first launch (fused) or one by one."""
        _check(lib().sol_network_set_layer_xr(self._h, C.c_int(layer), C.c_int(int(bool(fused)))))

    def fused_into(self, layer):
        """Index of the layer whose launch produces `layer`'s output (itself unless the plan fused it into
        the layer in front, as for the max pool behind a stem convolution)."""
        t = C.c_int(0)
        _check(lib().sol_network_layer_fused_into(self._h, C.c_int(layer), C.byref(t)))
        return t.value

    def concat_in_place(self, layer):
        """How many of the two inputs of concatenation layer `layer` their producers write in place (0..2)."""
        t = C.c_int(0)
        _check(lib().sol_network_concat_in_place(self._h, C.c_int(layer), C.byref(t)))
        return t.value

    def run_layer(self, layer, x, stream=None):
        """Runs one layer on whatever its producers left in the workspace (profiling aid)."""
        _check(lib().sol_network_run_layer(self._h, C.c_int(layer), _ptr(x), _ptr(self.y), _ptr(self.workspace),
                                           C.c_size_t(self.workspace.numel()), _stream(stream)))

    def layer_output(self, layer):
        """Output of an inner layer after a forward (network must keep its activations)."""
        d = self.output_desc(layer)
        p = C.c_void_p(0)
        _check(lib().sol_network_layer_output(self._h, C.c_int(layer), _ptr(self.workspace), C.byref(p)))
        off = p.value - self.workspace.data_ptr()
        nbytes = d.n * d.h * d.w * d.c * (2 if self.dt == BF16 else 4)
        return self.workspace[off:off + nbytes].view(torch_dtype(self.dt)).view(d.n, d.h, d.w, d.c)

    # ---- training step (networks created with NET_TRAINING)
    def backward(self, x, labels, stream=None):
        """Loss + full backward on what the last forward left; labels: int32 device tensor [n].
        Returns the device scalar holding the mean cross-entropy."""
        if not hasattr(self, "loss"):
            self.loss = torch.zeros(4, dtype=torch.float32, device=self.device)
        _check(lib().sol_network_backward(self._h, _ptr(x), _ptr(labels), _ptr(self.loss), _ptr(self.workspace),
                                          C.c_size_t(self.workspace.numel()), _stream(stream)))
        return self.loss[:1]

    def sgd_step(self, lr, momentum, stream=None):
        _check(lib().sol_network_sgd_step(self._h, C.c_float(lr), C.c_float(momentum), _stream(stream)))

    def tensor(self, layer, which):
        """fp32 view (inside the parameter buffer) of a layer's master parameter, gradient or batch statistic."""
        p, n = C.c_void_p(0), C.c_size_t(0)
        _check(lib().sol_network_tensor(self._h, C.c_int(layer), C.c_int(which), C.byref(p), C.byref(n)))
        off = p.value - self.param_buf.data_ptr()
        return self.param_buf[off:off + 4 * n.value].view(torch.float32)

    def layer_grad(self, layer):
        """Gradient w.r.t. a layer's output after a backward (NHWC, network dtype)."""
        return self._ws_view(layer, lib().sol_network_layer_grad)

    def layer_preact(self, layer):
        """Stored convolution output z of a conv+BN layer after a training forward (NHWC, network dtype)."""
        return self._ws_view(layer, lib().sol_network_layer_preact)

    def _ws_view(self, layer, fn):
        d = self.output_desc(layer)
        p = C.c_void_p(0)
        _check(fn(self._h, C.c_int(layer), _ptr(self.workspace), C.byref(p)))
        off = p.value - self.workspace.data_ptr()
        nbytes = d.n * d.h * d.w * d.c * (2 if self.dt == BF16 else 4)
        return self.workspace[off:off + nbytes].view(torch_dtype(self.dt)).view(d.n, d.h, d.w, d.c)

    def __del__(self):
        try:
            for g in getattr(self, "_graphs", []):
                lib().sol_graph_destroy(g)
            if self._h:
                lib().sol_network_destroy(self._h)
        except Exception:
            pass
