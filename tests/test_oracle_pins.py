"""Pins for the CPU checker: every layer definition is tied to something other than itself --
hand-worked numbers, closed forms, invariants, library routines of another code base (PyTorch's
CPU operators in fp64, the framework whose layer semantics the paper adopts, Sec. V), and
central finite differences for every backward function.  CPU only."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle as orc
from paper_2003_10688_amd import workloads as wl

R = np.random.default_rng(7)
T = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))  # noqa: E731


# ------------------------------------------------------------------------- conv forward
def test_conv_hand_worked():
    # 1 channel 3x3 input, 2x2 kernel, no pad, stride 1: four dot products done by hand.
    x = np.array([[1, 2, 3], [4, 5, 6], [7, 8, 9]], float).reshape(1, 1, 3, 3)
    w = np.array([[1, 0], [-1, 2]], float).reshape(1, 1, 2, 2)
    # y[p,q] = x[p,q] - x[p+1,q] + 2 x[p+1,q+1]   (correlation: no kernel flip)
    want = np.array([[1 - 4 + 10, 2 - 5 + 12], [4 - 7 + 16, 5 - 8 + 18]], float)
    got = orc.conv2d(x, w, np.array([0.5]))
    assert np.array_equal(got[0, 0], want + 0.5)
    # a flipped-kernel (true convolution) implementation would give x[p+1,q+1] - x[p,q+1] + 2 x[p,q]
    assert not np.array_equal(got[0, 0], np.array([[5 - 2 + 2, 6 - 3 + 4], [8 - 5 + 8, 9 - 6 + 10]]) + 0.5)


def test_conv_hand_worked_pad_stride_channels():
    # 2 input channels 2x2, one 3x3 kernel per channel, pad 1, stride 2 -> single output (p=q=0)
    x = np.array([[[1, 2], [3, 4]], [[10, 20], [30, 40]]], float).reshape(1, 2, 2, 2)
    w = np.arange(18, dtype=float).reshape(1, 2, 3, 3)
    # output (0,0) sees input rows/cols -1..1: taps (r,s) in {1,2}x{1,2} hit x[r-1,s-1]
    want = (1 * 4 + 2 * 5 + 3 * 7 + 4 * 8) + (10 * 13 + 20 * 14 + 30 * 16 + 40 * 17)
    got = orc.conv2d(x, w, None, (2, 2), (1, 1))
    assert got.shape == (1, 1, 1, 1) and got[0, 0, 0, 0] == want


def test_conv_delta_kernel_is_identity():
    x = R.standard_normal((2, 3, 6, 7))
    for k in (1, 3, 5):
        w = np.zeros((3, 3, k, k))
        for c in range(3):
            w[c, c, k // 2, k // 2] = 1.0
        assert np.array_equal(orc.conv2d(x, w, None, (1, 1), (k // 2, k // 2)), x)


def test_conv_1x1_is_matrix_product():
    x = R.standard_normal((2, 5, 4, 3))
    w = R.standard_normal((7, 5, 1, 1))
    want = np.einsum("nchw,kc->nkhw", x, w[:, :, 0, 0])
    assert np.allclose(orc.conv2d(x, w), want, rtol=1e-13, atol=1e-13)


def test_conv_ones_counts_taps():
    H, W, k, p = 5, 6, 3, 1
    y = orc.conv2d(np.ones((1, 2, H, W)), np.ones((1, 2, k, k)), None, (1, 1), (p, p))
    cnt_h = np.array([min(i + p, H - 1) - max(i - p, 0) + 1 for i in range(H)])
    cnt_w = np.array([min(j + p, W - 1) - max(j - p, 0) + 1 for j in range(W)])
    assert np.array_equal(y[0, 0], 2.0 * np.outer(cnt_h, cnt_w))


def test_conv_stride_is_subsampling_and_linear():
    x, x2 = R.standard_normal((1, 3, 9, 9)), R.standard_normal((1, 3, 9, 9))
    w = R.standard_normal((4, 3, 3, 3))
    y1 = orc.conv2d(x, w, None, (1, 1), (1, 1))
    y2 = orc.conv2d(x, w, None, (2, 2), (1, 1))
    assert np.array_equal(y2, y1[:, :, ::2, ::2])
    ysum = orc.conv2d(2.0 * x + x2, w, None, (1, 1), (1, 1))
    assert np.allclose(ysum, 2.0 * y1 + orc.conv2d(x2, w, None, (1, 1), (1, 1)), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("shape", [
    # N, C, H, W, K, R, S, sh, sw, ph, pw   (asymmetric on purpose: catches swapped axes)
    (2, 3, 8, 11, 4, 3, 3, 1, 1, 1, 1),
    (1, 4, 9, 7, 5, 3, 2, 2, 1, 1, 0),
    (2, 3, 15, 14, 6, 7, 7, 2, 2, 3, 3),
    (1, 8, 6, 6, 3, 1, 1, 2, 2, 0, 0),
    (1, 2, 7, 10, 3, 2, 5, 1, 3, 0, 2),
])
def test_conv_matches_library(shape):
    N, C, H, W, K, Rr, S, sh, sw, ph, pw = shape
    x, w, b = R.standard_normal((N, C, H, W)), R.standard_normal((K, C, Rr, S)), R.standard_normal(K)
    want = F.conv2d(T(x), T(w), T(b), stride=(sh, sw), padding=(ph, pw)).numpy()
    got = orc.conv2d(x, w, b, (sh, sw), (ph, pw))
    assert got.shape == want.shape
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
    # sampled evaluation agrees with the full one
    coords = np.stack([R.integers(0, d, 40) for d in got.shape], 1).astype(np.int32)
    pts = orc.conv2d_points(x, w, b, coords, (sh, sw), (ph, pw))
    assert np.array_equal(pts, got[tuple(coords.T)])


# ------------------------------------------------------------------------- depthwise conv
def test_dwconv_hand_worked():
    # 2 channels 3x3, one 2x2 filter each, no pad, stride 1: channels never mix.
    x = np.stack([np.arange(1, 10, dtype=float).reshape(3, 3), 10.0 * np.arange(1, 10, dtype=float).reshape(3, 3)])[None]
    w = np.array([[[1, 0], [-1, 2]], [[0, 1], [1, 0]]], float).reshape(2, 1, 2, 2)
    got = orc.dwconv2d(x, w, np.array([0.5, -1.0]))
    want0 = np.array([[1 - 4 + 10, 2 - 5 + 12], [4 - 7 + 16, 5 - 8 + 18]], float) + 0.5       # as in test_conv_hand_worked
    want1 = 10.0 * np.array([[2 + 4, 3 + 5], [5 + 7, 6 + 8]], float) - 1.0                      # x[p,q+1] + x[p+1,q]
    assert np.array_equal(got[0, 0], want0) and np.array_equal(got[0, 1], want1)


@pytest.mark.parametrize("shape", [(2, 5, 9, 8, 3, 3, 1, 1, 1, 1), (1, 7, 11, 6, 3, 3, 2, 2, 1, 1), (3, 4, 7, 7, 5, 3, 1, 2, 2, 0),
                                   (1, 3, 4, 4, 1, 1, 1, 1, 0, 0)])
def test_dwconv_is_block_diagonal_conv_and_matches_library(shape):
    N, C, H, W, Rr, S, sh, sw, ph, pw = shape
    x, w, b = R.standard_normal((N, C, H, W)), R.standard_normal((C, 1, Rr, S)), R.standard_normal(C)
    got = orc.dwconv2d(x, w, b, (sh, sw), (ph, pw))
    # the dense convolution (pinned above) whose weights are zero off the channel diagonal
    wf = np.zeros((C, C, Rr, S))
    for c in range(C):
        wf[c, c] = w[c, 0]
    assert np.allclose(got, orc.conv2d(x, wf, b, (sh, sw), (ph, pw)), rtol=1e-13, atol=1e-13)
    # the framework's grouped convolution with groups == channels
    want = F.conv2d(T(x), T(w), T(b), stride=(sh, sw), padding=(ph, pw), groups=C).numpy()
    assert got.shape == want.shape and np.allclose(got, want, rtol=1e-12, atol=1e-12)


def test_dwconv_delta_ones_and_fused_block():
    x = R.standard_normal((2, 6, 5, 7))
    d = np.zeros((6, 1, 3, 3))
    d[:, 0, 1, 1] = 1.0
    assert np.array_equal(orc.dwconv2d(x, d, None, (1, 1), (1, 1)), x)                    # delta filter: identity
    ones = orc.dwconv2d(np.ones((1, 2, 4, 5)), np.ones((2, 1, 3, 3)), None, (1, 1), (1, 1))
    assert ones[0, 0, 0, 0] == 4 and ones[0, 1, 0, 2] == 6 and ones[0, 0, 2, 2] == 9        # in-range taps at corner / edge / interior
    # fused block: depthwise conv -> explicit BN -> ReLU, composed from the pinned pieces
    l = wl.conv(6, 3, dw=True)
    prm = {"w": R.standard_normal((6, 1, 3, 3)), "bias": R.standard_normal(6), "gamma": R.uniform(0.5, 1.5, 6),
           "beta": R.uniform(-0.1, 0.1, 6), "mean": R.standard_normal(6) * 0.1, "var": R.uniform(0.5, 1.5, 6)}
    y, _, _ = orc.fused_conv(x, prm, l)
    want = orc.relu(orc.bn_infer(orc.dwconv2d(x, prm["w"], prm["bias"], (1, 1), (1, 1)), prm["gamma"], prm["beta"], prm["mean"], prm["var"]))
    assert np.array_equal(y, want)


# ------------------------------------------------------------------------------- channel concatenation
def test_concat_placement_linearity_and_in_a_network():
    a = np.array([1.0, 2.0]).reshape(1, 2, 1, 1)
    b = np.array([3.0]).reshape(1, 1, 1, 1)
    assert orc.concat(a, b).ravel().tolist() == [1.0, 2.0, 3.0] and orc.concat(b, a).ravel().tolist() == [3.0, 1.0, 2.0]
    a, b = R.standard_normal((2, 3, 4, 5)), R.standard_normal((2, 2, 4, 5))
    c = orc.concat(a, b)
    assert np.array_equal(c, torch.cat([T(a), T(b)], 1).numpy())                      # the library's routine
    # a 1x1 convolution of a concatenation is the sum of the 1x1 convolutions of its parts with the split filter
    w = R.standard_normal((4, 5, 1, 1))
    whole = orc.conv2d(c, w, None, (1, 1), (0, 0))
    parts = orc.conv2d(a, w[:, :3], None, (1, 1), (0, 0)) + orc.conv2d(b, w[:, 3:], None, (1, 1), (0, 0))
    assert np.allclose(whole, parts, rtol=1e-13, atol=1e-13)
    with pytest.raises(ValueError):
        orc.concat(a, R.standard_normal((2, 2, 4, 6)))
    # inside a layer list: a fire module equals its pieces composed by hand
    layers = wl.fire_layers(0, -1, 4, 6)
    prm = wl.make_params(layers, 3, 77, bias_std=0.3)
    x = R.standard_normal((2, 3, 6, 6))
    outs, _ = orc.network_forward(layers, prm, x, return_all=True)
    sq = orc.relu(orc.conv2d(x, prm[0]["w"], prm[0]["bias"], (1, 1), (0, 0)))
    e1 = orc.relu(orc.conv2d(sq, prm[1]["w"], prm[1]["bias"], (1, 1), (0, 0)))
    e3 = orc.relu(orc.conv2d(sq, prm[2]["w"], prm[2]["bias"], (1, 1), (1, 1)))
    assert outs[3].shape == (2, 12, 6, 6)
    assert np.array_equal(outs[3][:, :6], e1) and np.array_equal(outs[3][:, 6:], e3)


def test_squeezenet_shaped_list_is_wired_like_the_published_network():
    """Channel counts after every fire module and the classifier, as published for SqueezeNet 1.1."""
    L = wl.squeezenet_layers()
    ch = wl.layer_channels(L, 3)
    joins = [ch[i] for i, l in enumerate(L) if l["kind"] == "concat"]
    assert joins == [128, 128, 256, 256, 384, 384, 512, 512]
    assert sum(l["kind"] == "pool" for l in L) == 3 and ch[-1] == 1000 and L[-1]["kind"] == "gap"
    for i, l in enumerate(L):
        if l["kind"] == "concat":                        # both inputs are the expand convolutions of one squeeze layer
            assert L[l["src"]]["src"] == L[l["res"]]["src"] == l["src"] - 1
            assert (L[l["src"]]["kh"], L[l["res"]]["kh"]) == (1, 3)


# ------------------------------------------------------------------------------- BN, ReLU
def test_bn_identity_and_affine():
    x = R.standard_normal((2, 3, 4, 4))
    one, zero = np.ones(3), np.zeros(3)
    y = orc.bn_infer(x, one, zero, zero, one - 1e-5, 1e-5)
    assert np.allclose(y, x, rtol=1e-15, atol=1e-15)
    g, b, m, v = R.uniform(0.5, 1.5, 3), R.uniform(-1, 1, 3), R.standard_normal(3), R.uniform(0.5, 1.5, 3)
    y = orc.bn_infer(x, g, b, m, v, 1e-5)
    scale = g / np.sqrt(v + 1e-5)                 # folded form == explicit form
    want = x * scale[None, :, None, None] + (b - m * scale)[None, :, None, None]
    assert np.allclose(y, want, rtol=1e-13, atol=1e-13)
    want_lib = F.batch_norm(T(x), T(m), T(v), T(g), T(b), False, 0.0, 1e-5).numpy()
    assert np.allclose(y, want_lib, rtol=1e-13, atol=1e-13)


def test_bn_train_statistics():
    x = R.standard_normal((4, 3, 5, 5)) * 3 + 2
    y, mean, var = orc.bn_train(x, np.ones(3), np.zeros(3), 1e-5)
    assert np.allclose(mean, x.mean((0, 2, 3))) and np.allclose(var, x.var((0, 2, 3)))  # biased var
    assert np.allclose(y.mean((0, 2, 3)), 0, atol=1e-13)
    assert np.allclose(y.var((0, 2, 3)), var / (var + 1e-5), rtol=1e-12)
    g, b = R.uniform(0.5, 1.5, 3), R.uniform(-1, 1, 3)
    y2, _, _ = orc.bn_train(x, g, b, 1e-5)
    want = F.batch_norm(T(x), None, None, T(g), T(b), True, 0.0, 1e-5).numpy()
    assert np.allclose(y2, want, rtol=1e-12, atol=1e-12)


def test_relu_properties():
    x = R.standard_normal(1000)
    y = orc.relu(x)
    assert np.array_equal(orc.relu(y), y)                       # idempotent
    assert np.array_equal(y - orc.relu(-x), x)                  # relu(x) - relu(-x) = x
    assert y.min() == 0.0 and np.array_equal(y[x > 0], x[x > 0])


# ---------------------------------------------------------------------------------- pools
def test_maxpool_hand_worked_and_ties():
    x = np.array([[1, 5, 2, 2], [5, 0, 2, 2], [-1, -2, -3, -4], [-2, -1, -4, -3]], float).reshape(1, 1, 4, 4)
    y, a = orc.maxpool(x, (2, 2), (2, 2), (0, 0))
    assert np.array_equal(y[0, 0], [[5, 2], [-1, -3]])
    # ties: the first element in row-major window order wins; index is ih*W+iw in the input plane
    assert np.array_equal(a[0, 0], [[1, 2], [8, 10]])


def test_maxpool_constant_ramp_and_relu_commute():
    c = np.full((1, 2, 6, 6), 3.25)
    for k, s, p in ((2, 2, 0), (3, 2, 1), (3, 1, 1)):
        y, a = orc.maxpool(c, (k, k), (s, s), (p, p))
        assert np.all(y == 3.25)
        ya = orc.avgpool(c, (k, k), (s, s), (p, p), count_pad=False)
        assert np.allclose(ya, 3.25, rtol=1e-15)
    up = np.arange(36, dtype=float).reshape(1, 1, 6, 6)
    _, a = orc.maxpool(up, (2, 2), (2, 2), (0, 0))
    assert np.array_equal(a[0, 0], [[7, 9, 11], [19, 21, 23], [31, 33, 35]])     # last element of window
    _, a = orc.maxpool(-up, (2, 2), (2, 2), (0, 0))
    assert np.array_equal(a[0, 0], [[0, 2, 4], [12, 14, 16], [24, 26, 28]])      # first element of window
    # ReLU and max-pool commute (the paper's graph rewrite, Sec. III-A); also with -inf padding
    x = R.standard_normal((2, 3, 9, 9))
    for k, s, p in ((2, 2, 0), (3, 2, 1)):
        assert np.array_equal(orc.maxpool(orc.relu(x), (k, k), (s, s), (p, p))[0],
                              orc.relu(orc.maxpool(x, (k, k), (s, s), (p, p))[0]))


@pytest.mark.parametrize("cfg", [(2, 2, 2, 2, 0, 0), (3, 3, 2, 2, 1, 1), (3, 2, 1, 2, 1, 0), (2, 3, 2, 1, 0, 1)])
def test_pools_match_library(cfg):
    kh, kw, sh, sw, ph, pw = cfg
    x = np.round(R.standard_normal((2, 3, 9, 8)) * 2) / 2          # coarse grid -> many exact ties
    y, a = orc.maxpool(x, (kh, kw), (sh, sw), (ph, pw))
    wy, wa = F.max_pool2d(T(x), (kh, kw), (sh, sw), (ph, pw), return_indices=True)
    assert np.array_equal(y, wy.numpy()) and np.array_equal(a, wa.numpy().astype(np.int32))
    # argmax points at an element equal to the output, and nothing earlier in the plane-order ties it
    flat = x.reshape(2, 3, -1)
    assert np.array_equal(np.take_along_axis(flat, a.reshape(2, 3, -1).astype(np.int64), 2).reshape(y.shape), y)
    for cp in (True, False):
        ya = orc.avgpool(x, (kh, kw), (sh, sw), (ph, pw), cp)
        wa_ = F.avg_pool2d(T(x), (kh, kw), (sh, sw), (ph, pw), count_include_pad=cp).numpy()
        assert np.allclose(ya, wa_, rtol=1e-13, atol=1e-13)


def test_avgpool_paper_listing_shape_and_ramp():
    # the paper's pooling listing: 3x3 window, stride 1, divide by 9 (Sec. IV, AveragePooling listing),
    # replayed on a linear ramp: the window mean of a ramp is the ramp at the window centre.
    H = W = 16
    ii, jj = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    ramp = (2.0 * ii + 0.5 * jj + 1.0).reshape(1, 1, H, W)
    y = orc.avgpool(ramp, (3, 3), (1, 1), (0, 0), True)
    assert y.shape == (1, 1, H - 2, W - 2)
    assert np.allclose(y[0, 0], ramp[0, 0, 1:-1, 1:-1], rtol=1e-14)
    # count-padding switch changes only the border outputs
    a = orc.avgpool(ramp, (3, 3), (1, 1), (1, 1), True)
    b = orc.avgpool(ramp, (3, 3), (1, 1), (1, 1), False)
    assert np.array_equal(a[0, 0, 1:-1, 1:-1], b[0, 0, 1:-1, 1:-1])
    assert np.allclose(a[0, 0, 0, 0] * 9, b[0, 0, 0, 0] * 4, rtol=1e-14)
    assert np.allclose(orc.gap(ramp)[0, 0], ramp.mean(), rtol=1e-14)


# ------------------------------------------------------------------------- linear, bf16
def test_linear():
    x = R.standard_normal((3, 6))
    assert np.array_equal(orc.linear(x, np.eye(6)), x)
    w, b = R.standard_normal((4, 6)), R.standard_normal(4)
    assert np.allclose(orc.linear(x, w, b), x @ w.T + b, rtol=1e-13, atol=1e-13)
    # equals a 1x1 convolution on a 1x1 image; weight layout [Out][In] vs [In][Out] is only storage
    assert np.allclose(orc.linear(x, w, b), orc.conv2d(x.reshape(3, 6, 1, 1), w.reshape(4, 6, 1, 1), b)[:, :, 0, 0])
    assert np.allclose(orc.linear(x, w, b), (np.ascontiguousarray(w.T).T @ x.T).T + b)


def test_bf16_rounding():
    e = 2.0 ** -8
    assert orc.bf16(1.0 + e) == 1.0                      # tie -> even (mantissa 0)
    assert orc.bf16(1.0 + 3 * e) == 1.0 + 4 * e          # tie -> even (mantissa 2)
    assert orc.bf16(1.0 + 1.0001 * e) == 1.0 + 2 * e     # just above the tie
    assert orc.bf16(-(1.0 + 3 * e)) == -(1.0 + 4 * e)
    assert orc.bf16(255.0) == 255.0 and orc.bf16(257.0) == 256.0 and orc.bf16(259.0) == 260.0
    assert orc.bf16(2.0 ** -133) == 2.0 ** -133          # smallest subnormal survives
    assert orc.bf16(2.0 ** -134) == 0.0                  # tie to even (zero)
    assert orc.bf16(1.5 * 2.0 ** -133) == 2.0 ** -132
    assert orc.bf16(3.4e38) == math.inf and orc.bf16(-3.4e38) == -math.inf
    big = float.fromhex("0x1.FEp127")
    assert orc.bf16(big) == big
    assert math.isnan(orc.bf16(math.nan)) and orc.bf16(math.inf) == math.inf
    # against the tensor library's converter on fp32-representable values (no double rounding there)
    v = (R.standard_normal(20000) * np.exp(R.uniform(-20, 20, 20000))).astype(np.float32)
    want = torch.from_numpy(v).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(orc.round_bf16(v.astype(np.float64)), want)
    # bf16 x bf16 products are exact in fp32/fp64: a short dot product of bf16 values has a closed form
    a = orc.round_bf16(R.standard_normal(8))
    assert orc.conv2d(a.reshape(1, 8, 1, 1), a.reshape(1, 8, 1, 1))[0, 0, 0, 0] == math.fsum(a * a)


# ------------------------------------------------------------------- fused block, network
def test_fused_block_and_residual():
    l = {"kind": "conv", "cout": 4, "kh": 3, "kw": 3, "sh": 1, "sw": 1, "ph": 1, "pw": 1, "bn": True,
         "act": "relu", "pool": {"kind": "max", "kh": 2, "kw": 2, "sh": 2, "sw": 2, "ph": 0, "pw": 0}}
    x = R.standard_normal((2, 3, 8, 8))
    p = {"w": R.standard_normal((4, 3, 3, 3)), "bias": R.standard_normal(4), "gamma": R.uniform(0.5, 1.5, 4),
         "beta": R.uniform(-0.1, 0.1, 4), "mean": R.standard_normal(4) * 0.1, "var": R.uniform(0.5, 1.5, 4)}
    res = R.standard_normal((2, 4, 8, 8))
    y, arg, pre = orc.fused_conv(x, p, l, res, want_prepool=True)
    t = F.conv2d(T(x), T(p["w"]), T(p["bias"]), padding=1)
    t = F.batch_norm(t, T(p["mean"]), T(p["var"]), T(p["gamma"]), T(p["beta"]), False, 0.0, 1e-5)
    t = F.relu(t + T(res))
    assert np.allclose(pre, t.numpy(), rtol=1e-12, atol=1e-12)
    wy, wa = F.max_pool2d(t, 2, 2, return_indices=True)
    assert np.allclose(y, wy.numpy(), rtol=1e-12, atol=1e-12) and np.array_equal(arg, wa.numpy())
    # zero weights: block output is relu(shift + residual)
    p0 = dict(p, w=np.zeros_like(p["w"]), bias=np.zeros(4))
    l0 = dict(l, pool=None, bn=False, act="none")
    assert np.array_equal(orc.fused_conv(x, p0, l0, res)[0], res)


def test_bn_points_and_fused_block_points_agree_with_the_full_tensors():
    """The sampled evaluations used against full-size GPU outputs: bn_infer_points is the pinned per-channel map at
    scattered elements (library batch-norm and the folded affine form as independent references), and
    fused_conv_points equals the pinned full fused block at random coordinates -- with residual, ReLU, stride,
    padding and the bf16 store -- exactly."""
    g, b, m, v = R.uniform(0.5, 1.5, 5), R.uniform(-1, 1, 5), R.standard_normal(5), R.uniform(0.5, 1.5, 5)
    x = R.standard_normal((3, 5, 4, 6))
    full = orc.bn_infer(x, g, b, m, v, 1e-5)
    coords = np.stack([R.integers(0, d, 60) for d in x.shape], 1).astype(np.int32)
    pts = orc.bn_infer_points(x[tuple(coords.T)], coords[:, 1], g, b, m, v, 1e-5)
    assert np.array_equal(pts, full[tuple(coords.T)])
    lib = F.batch_norm(T(x), T(m), T(v), T(g), T(b), False, 0.0, 1e-5).numpy()
    assert np.allclose(pts, lib[tuple(coords.T)], rtol=1e-13, atol=1e-13)
    scale = g / np.sqrt(v + 1e-5)
    assert np.allclose(pts, x[tuple(coords.T)] * scale[coords[:, 1]] + (b - m * scale)[coords[:, 1]], rtol=1e-13, atol=1e-13)
    # a wrong channel index (e.g. the batch index used as channel) must show: channels differ in every parameter
    assert not np.allclose(orc.bn_infer_points(x[tuple(coords.T)], coords[:, 0], g, b, m, v, 1e-5), full[tuple(coords.T)])

    for (k, sh, ph, bn, act, with_res, bf) in [(3, 1, 1, True, "relu", True, False), (1, 2, 0, True, "none", False, True),
                                               (3, 2, 1, False, "relu", True, True), (5, 1, 2, True, "relu", False, False)]:
        l = {"kind": "conv", "cout": 6, "kh": k, "kw": k, "sh": sh, "sw": sh, "ph": ph, "pw": ph, "bn": bn, "act": act, "pool": None}
        xx = orc.round_bf16(R.standard_normal((2, 4, 9, 11))) if bf else R.standard_normal((2, 4, 9, 11))
        p = {"w": R.standard_normal((6, 4, k, k)), "bias": R.standard_normal(6), "gamma": R.uniform(0.5, 1.5, 6),
             "beta": R.uniform(-0.1, 0.1, 6), "mean": R.standard_normal(6) * 0.1, "var": R.uniform(0.5, 1.5, 6)}
        ho, wo = orc.out_size(9, k, sh, ph), orc.out_size(11, k, sh, ph)
        res = R.standard_normal((2, 6, ho, wo)) if with_res else None
        full, _, _ = orc.fused_conv(xx, p, l, res, bf16=bf)
        assert full.shape == (2, 6, ho, wo)
        cs = np.stack([R.integers(0, d, 80) for d in full.shape], 1).astype(np.int32)
        got = orc.fused_conv_points(xx, p, l, cs, res, bf16=bf)
        assert np.array_equal(got, full[tuple(cs.T)])
        if bf:
            assert np.array_equal(got, orc.round_bf16(got))          # stored values are bf16 numbers
        # against the library composition (not through the checker's own full-tensor code)
        t = F.conv2d(T(xx), T(p["w"]), T(p["bias"]), stride=sh, padding=ph)
        if bn:
            t = F.batch_norm(t, T(p["mean"]), T(p["var"]), T(p["gamma"]), T(p["beta"]), False, 0.0, 1e-5)
        if with_res:
            t = t + T(res)
        if act == "relu":
            t = F.relu(t)
        tol = 2.0 ** -7 if bf else 1e-12
        assert np.allclose(got, t.numpy()[tuple(cs.T)], rtol=tol, atol=tol * 1e-3 if bf else tol)


def test_pre_activation_block_and_densenet_shaped_list():
    """Input-side BN + ReLU of a convolution (pre-activation order): equals the tensor library's composition; the zero
    padding applies to the ACTIVATED tensor (a positive BN shift must not leak into the border taps); points version
    agrees; in bf16 mode the activated tensor is a rounding point.  The DenseNet-shaped list is wired like the
    published network (channel counts per block, 120 convolutions + the final BN-ReLU)."""
    l = wl.conv(5, 3, pre_bn=True)
    x = R.standard_normal((2, 4, 7, 6))
    p = {"w": R.standard_normal((5, 4, 3, 3)), "bias": R.standard_normal(5), "gamma": R.uniform(0.5, 1.5, 5), "beta": R.uniform(-0.1, 0.1, 5),
         "mean": R.standard_normal(5) * 0.1, "var": R.uniform(0.5, 1.5, 5), "pre_gamma": R.uniform(0.5, 1.5, 4),
         "pre_beta": R.uniform(0.5, 1.0, 4), "pre_mean": R.standard_normal(4) * 0.1, "pre_var": R.uniform(0.5, 1.5, 4)}
    y, _, _ = orc.fused_conv(x, p, l)
    a = F.relu(F.batch_norm(T(x), T(p["pre_mean"]), T(p["pre_var"]), T(p["pre_gamma"]), T(p["pre_beta"]), False, 0.0, 1e-5))
    t = F.conv2d(a, T(p["w"]), T(p["bias"]), padding=1)
    t = F.relu(F.batch_norm(t, T(p["mean"]), T(p["var"]), T(p["gamma"]), T(p["beta"]), False, 0.0, 1e-5))
    assert np.allclose(y, t.numpy(), rtol=1e-12, atol=1e-12)
    # activating a zero-padded input instead gives relu(pre_beta - ...) > 0 in the border taps: visibly different
    xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (1, 1)))
    wrong, _, _ = orc.fused_conv(xp, p, dict(l, ph=0, pw=0))
    assert wrong.shape == y.shape and not np.allclose(wrong[:, :, 0, :], y[:, :, 0, :], rtol=1e-3, atol=1e-3)
    assert np.allclose(wrong[:, :, 2:-2, 2:-2], y[:, :, 2:-2, 2:-2], rtol=1e-12, atol=1e-12)          # interior: same
    # bf16 mode: the activated tensor is rounded, then the output
    xb = orc.round_bf16(x)
    yb, _, _ = orc.fused_conv(xb, p, l, bf16=True)
    ab = orc.round_bf16(a.numpy() if False else F.relu(F.batch_norm(T(xb), T(p["pre_mean"]), T(p["pre_var"]), T(p["pre_gamma"]), T(p["pre_beta"]),
                                                                False, 0.0, 1e-5)).numpy())
    tb = F.conv2d(T(ab), T(p["w"]), T(p["bias"]), padding=1)
    tb = F.relu(F.batch_norm(tb, T(p["mean"]), T(p["var"]), T(p["gamma"]), T(p["beta"]), False, 0.0, 1e-5)).numpy()
    assert np.allclose(yb, orc.round_bf16(tb), rtol=2.0 ** -7, atol=1e-6) and np.array_equal(yb, orc.round_bf16(yb))

    L = wl.densenet_layers()
    ch = wl.layer_channels(L, 3)
    convs = [l for l in L if l["kind"] == "conv" and not l.get("dw")]
    assert len(convs) == 120 and sum(1 for l in L if l["kind"] == "concat") == 58
    ends = [ch[i - 1] for i, l in enumerate(L) if l["kind"] == "conv" and l.get("pool")]            # features entering a transition
    assert ends == [256, 512, 1024] and ch[-3] == 1024 and ch[-1] == 1000
    wk = wl.config(8, batch=2, hw=32)
    outs, _ = orc.network_forward(wk.layers, wk.params, wk.x, return_all=True)
    assert outs[-1].shape == (2, 1000) and outs[1].shape == (2, 64, 8, 8)
    i = next(i for i, l in enumerate(wk.layers) if l["kind"] == "concat")
    assert np.array_equal(outs[i][:, :64], outs[1]) and np.array_equal(outs[i][:, 64:], outs[i - 1])   # concat appends the new features


def test_network_is_composition_and_batch_permutes():
    from paper_2003_10688_amd import workloads as wl

    wk = wl.config(1, batch=3, hw=8)
    outs, args = orc.network_forward(wk.layers, wk.params, wk.x, return_all=True)
    assert [o.shape for o in outs] == [(3, 32, 8, 8), (3, 32, 4, 4), (3, 64, 4, 4), (3, 64, 2, 2), (3, 64), (3, 10)]
    assert args[1].dtype == np.int32 and args[0] is None
    # same chain through the other code base's operators
    t = T(wk.x)
    for l, p in zip(wk.layers[:4], wk.params[:4]):
        t = F.conv2d(t, T(p["w"]), T(p["bias"]), padding=1)
        t = F.relu(F.batch_norm(t, T(p["mean"]), T(p["var"]), T(p["gamma"]), T(p["beta"]), False, 0.0, 1e-5))
        if l["pool"]:
            t = F.max_pool2d(t, 2, 2)
    t = F.linear(t.mean((2, 3)), T(wk.params[5]["w"]), T(wk.params[5]["bias"]))
    assert np.allclose(outs[-1], t.numpy(), rtol=1e-11, atol=1e-11)
    perm = [2, 0, 1]
    assert np.allclose(orc.network_forward(wk.layers, wk.params, wk.x[perm]), outs[-1][perm], rtol=1e-13)


def test_resnet_shapes_and_residual_wiring():
    from paper_2003_10688_amd import workloads as wl

    wk = wl.config(3, batch=1, hw=32)
    assert sum(l["kind"] == "conv" for l in wk.layers) == 53
    outs = orc.network_forward(wk.layers, wk.params, wk.x, bf16=True, return_all=True)[0]
    assert outs[0].shape == (1, 64, 16, 16) and outs[1].shape == (1, 64, 8, 8)
    assert outs[-3].shape == (1, 2048, 1, 1) and outs[-1].shape == (1, 1000)
    assert np.array_equal(orc.round_bf16(outs[-1]), outs[-1])       # every stored value is a bf16 number
    wk18 = wl.config(2, batch=1, hw=32)
    assert sum(l["kind"] == "conv" for l in wk18.layers) == 20
    o18 = orc.network_forward(wk18.layers, wk18.params, wk18.x, bf16=True, return_all=True)[0]
    assert o18[-3].shape == (1, 512, 1, 1)
    # the library's own ResNet-18-shaped forward with the same tensors (fp64, no bf16 rounding)
    o = orc.network_forward(wk18.layers, wk18.params, wk18.x, return_all=True)[0]
    t = _torch_forward(wk18.layers, wk18.params, T(wk18.x))
    assert np.allclose(o[-1], t.numpy(), rtol=1e-9, atol=1e-9)


def _torch_forward(layers, params, x):
    outs = []
    for i, (l, p) in enumerate(zip(layers, params)):
        s = l.get("src", -1)
        t = (x if i == 0 else outs[i - 1]) if s == -1 else outs[s]
        if l["kind"] == "conv":
            t = F.conv2d(t, T(p["w"]), T(p["bias"]), stride=(l["sh"], l["sw"]), padding=(l["ph"], l["pw"]))
            if l["bn"]:
                t = F.batch_norm(t, T(p["mean"]), T(p["var"]), T(p["gamma"]), T(p["beta"]), False, 0.0, 1e-5)
            if l["res"] >= 0:
                t = t + outs[l["res"]]
            if l["act"] == "relu":
                t = F.relu(t)
            if l["pool"]:
                pd = l["pool"]
                t = F.max_pool2d(t, (pd["kh"], pd["kw"]), (pd["sh"], pd["sw"]), (pd["ph"], pd["pw"]))
        elif l["kind"] == "pool":
            pd = l["pool"]
            t = F.max_pool2d(t, (pd["kh"], pd["kw"]), (pd["sh"], pd["sw"]), (pd["ph"], pd["pw"]))
        elif l["kind"] == "gap":
            t = t.mean((2, 3))
        else:
            t = F.linear(t, T(p["w"]), T(p["bias"]))
        outs.append(t)
    return outs[-1]


# ------------------------------------------------------------------------------ backward
def _fd(f, x, h=1e-5):
    """Central finite-difference gradient of scalar f at x."""
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + h
        fp = f(x)
        x[i] = old - h
        fm = f(x)
        x[i] = old
        g[i] = (fp - fm) / (2 * h)
    return g


def test_conv_backward_fd_and_library():
    x, w = R.standard_normal((2, 2, 5, 6)), R.standard_normal((3, 2, 3, 2))
    st, pd = (2, 1), (1, 0)
    gy = R.standard_normal(orc.conv2d(x, w, None, st, pd).shape)
    dx = orc.conv2d_dgrad(gy, w, x.shape, st, pd)
    dw, db = orc.conv2d_wgrad(x, gy, w.shape, st, pd)
    assert np.allclose(dx, _fd(lambda a: (orc.conv2d(a, w, None, st, pd) * gy).sum(), x.copy()), rtol=1e-6, atol=1e-7)
    assert np.allclose(dw, _fd(lambda a: (orc.conv2d(x, a, None, st, pd) * gy).sum(), w.copy()), rtol=1e-6, atol=1e-7)
    assert np.allclose(db, gy.sum((0, 2, 3)))
    tx, tw = T(x).requires_grad_(), T(w).requires_grad_()
    (F.conv2d(tx, tw, None, st, pd) * T(gy)).sum().backward()
    assert np.allclose(dx, tx.grad.numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(dw, tw.grad.numpy(), rtol=1e-12, atol=1e-12)
    # delta input: wgrad closed form -- dw[k,c,r,s] picks one dy element per tap
    xd = np.zeros((1, 1, 5, 5)); xd[0, 0, 2, 2] = 1.0
    gy = R.standard_normal((1, 1, 5, 5))
    dw, _ = orc.conv2d_wgrad(xd, gy, (1, 1, 3, 3), (1, 1), (1, 1))
    assert np.array_equal(dw[0, 0], gy[0, 0, 1:4, 1:4][::-1, ::-1])


def test_bn_backward_fd_library_and_invariants():
    x = R.standard_normal((3, 2, 4, 3)) * 2 + 1
    g, b = R.uniform(0.5, 1.5, 2), R.uniform(-1, 1, 2)
    gy = R.standard_normal(x.shape)
    _, mean, var = orc.bn_train(x, g, b, 1e-5)
    dx, dg, dbt = orc.bn_train_bwd(x, gy, g, mean, var, 1e-5)
    f = lambda a: (orc.bn_train(a, g, b, 1e-5)[0] * gy).sum()  # noqa: E731  (through the batch statistics)
    assert np.allclose(dx, _fd(f, x.copy()), rtol=1e-5, atol=1e-7)
    assert np.allclose(dg, _fd(lambda a: (orc.bn_train(x, a, b, 1e-5)[0] * gy).sum(), g.copy()), rtol=1e-6)
    assert np.allclose(dbt, gy.sum((0, 2, 3)))
    xh = (x - mean[None, :, None, None]) / np.sqrt(var + 1e-5)[None, :, None, None]
    assert np.allclose(dx.sum((0, 2, 3)), 0, atol=1e-12)
    # sum(dx*xhat) = gamma/sigma * dgamma * eps/(var+eps): zero up to the eps inside the square root
    assert np.allclose((dx * xh).sum((0, 2, 3)), g / np.sqrt(var + 1e-5) * dg * 1e-5 / (var + 1e-5), atol=1e-11)
    tx, tg, tb = T(x).requires_grad_(), T(g).requires_grad_(), T(b).requires_grad_()
    (F.batch_norm(tx, None, None, tg, tb, True, 0.0, 1e-5) * T(gy)).sum().backward()
    assert np.allclose(dx, tx.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dg, tg.grad.numpy(), rtol=1e-10)


def test_pool_relu_gap_linear_backward():
    x = R.standard_normal((2, 2, 7, 6))
    y, a = orc.maxpool(x, (3, 3), (2, 2), (1, 1))
    gy = R.standard_normal(y.shape)
    dx = orc.maxpool_bwd(gy, a, x.shape)
    assert np.isclose(dx.sum(), gy.sum())                                    # gradient mass conserved
    tx = T(x).requires_grad_()
    (F.max_pool2d(tx, 3, 2, 1) * T(gy)).sum().backward()
    assert np.allclose(dx, tx.grad.numpy(), rtol=1e-13, atol=1e-13)          # overlapping windows accumulate
    for cp in (True, False):
        dxa = orc.avgpool_bwd(gy, x.shape, (3, 3), (2, 2), (1, 1), cp)
        tx = T(x).requires_grad_()
        (F.avg_pool2d(tx, 3, 2, 1, count_include_pad=cp) * T(gy)).sum().backward()
        assert np.allclose(dxa, tx.grad.numpy(), rtol=1e-13, atol=1e-13)
    yr = orc.relu(x)
    g2 = R.standard_normal(x.shape)
    assert np.array_equal(orc.relu_bwd(yr, g2), np.where(x > 0, g2, 0.0))
    gg = R.standard_normal((2, 2))
    assert np.allclose(orc.gap_bwd(gg, x.shape), np.broadcast_to(gg[:, :, None, None] / 42.0, x.shape))
    xl, wl_, gl = R.standard_normal((3, 5)), R.standard_normal((4, 5)), R.standard_normal((3, 4))
    dxl, dwl, dbl = orc.linear_bwd(xl, wl_, gl)
    assert np.allclose(dxl, gl @ wl_) and np.allclose(dwl, gl.T @ xl) and np.allclose(dbl, gl.sum(0))


def test_softmax_ce_and_sgd():
    loss, dz = orc.softmax_ce(np.zeros((4, 1000)), np.array([0, 5, 999, 17]))
    assert abs(loss - math.log(1000.0)) < 1e-12                              # uniform logits -> ln K
    z, lab = R.standard_normal((5, 7)) * 3, R.integers(0, 7, 5)
    loss, dz = orc.softmax_ce(z, lab)
    assert np.allclose(dz.sum(1), 0, atol=1e-15)
    assert np.allclose(dz, _fd(lambda a: orc.softmax_ce(a, lab, False)[0], z.copy()), rtol=1e-6, atol=1e-9)
    assert np.isclose(loss, F.cross_entropy(T(z), torch.from_numpy(lab).long()).item(), rtol=1e-13)
    big, _ = orc.softmax_ce(z + 1000.0, lab)                                  # shift invariance / no overflow
    assert np.isclose(big, loss, rtol=1e-10)
    w0 = R.standard_normal(10); w, v, g = w0.copy(), np.zeros(10), R.standard_normal(10)
    orc.sgd(w, v, g, 0.1, 0.9)
    assert np.allclose(w, w0 - 0.1 * g) and np.array_equal(v, g)             # first step closed form
    g2 = R.standard_normal(10)
    orc.sgd(w, v, g2, 0.1, 0.9)
    assert np.allclose(v, 0.9 * g + g2) and np.allclose(w, w0 - 0.1 * g - 0.1 * (0.9 * g + g2))


# ------------------------------------------------------------------------ training step
def _tiny_resnet():
    L = [wl.conv(8, 3, s=2, p=1), wl.pool("max", 3, 2, 1), wl.conv(8, 3, src=1),
         wl.conv(16, 1, s=2, p=0, act="none", src=1), wl.conv(16, 3, s=2, src=2, res=3), wl.gap(), wl.linear(5)]
    P = wl.make_params(L, 3, 123, bias_std=0.0)
    return L, P


def test_train_step_matches_autograd():
    """Unrounded training step (batch-stat BN, residual, overlapping max pool, strided convs, CE loss)
    against torch autograd in fp64: loss, every gradient, and the SGD-with-momentum update."""
    import torch.nn.functional as F
    L, P = _tiny_resnet()
    x = wl.make_input((4, 3, 17, 19), 5)
    lab = np.array([0, 3, 4, 1])
    T = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    out = orc.network_train_step(L, P, x, lab, 0.1, 0.9)
    tp = [{k: T(v).requires_grad_() for k, v in p.items() if isinstance(v, np.ndarray)} for p in P]
    outs = []
    for i, (l, p) in enumerate(zip(L, tp)):
        s = l.get("src", -1)
        t = (T(x) if i == 0 else outs[i - 1]) if s == -1 else outs[s]
        if l["kind"] == "conv":
            y = F.conv2d(t, p["w"], p["bias"], stride=(l["sh"], l["sw"]), padding=(l["ph"], l["pw"]))
            if l["bn"]:
                y = F.batch_norm(y, None, None, p["gamma"], p["beta"], True, 0.0, 1e-5)
            if l["res"] >= 0:
                y = y + outs[l["res"]]
            if l["act"] == "relu":
                y = F.relu(y)
        elif l["kind"] == "pool":
            y = F.max_pool2d(t, 3, 2, 1)
        elif l["kind"] == "gap":
            y = t.mean((2, 3))
        else:
            y = F.linear(t, p["w"], p["bias"])
        outs.append(y)
    loss = F.cross_entropy(outs[-1], torch.from_numpy(lab).long())
    loss.backward()
    assert abs(out["loss"] - loss.item()) < 1e-12
    for i, (g, p) in enumerate(zip(out["grads"], tp)):
        for k, v in g.items():
            ref = p[k].grad.numpy()
            assert np.abs(v - ref).max() <= 1e-12 * max(np.abs(ref).max(), 1.0), (i, k)
            # first step from zero velocity: w1 = w0 - lr g ; second step uses v = mu g + g2
            np.testing.assert_allclose(out["new_params"][i][k], p[k].detach().numpy() - 0.1 * ref, atol=1e-12)
    out2 = orc.network_train_step(L, out["new_params"], x, lab, 0.1, 0.9, velocity=out["velocity"])
    i, k = 2, "w"
    v2 = 0.9 * out["grads"][i][k] + out2["grads"][i][k]
    np.testing.assert_allclose(out2["new_params"][i][k], out["new_params"][i][k] - 0.1 * v2, atol=1e-12)


def test_train_step_bf16_rounding_points():
    """bf16 mode: every stored tensor lies on the bf16 grid, statistics and weight gradients do not."""
    L, P = _tiny_resnet()
    x = wl.to_bf16_grid(wl.make_input((4, 3, 17, 19), 5))
    out = orc.network_train_step(L, P, x, np.array([0, 3, 4, 1]), 0.1, 0.9, bf16=True)
    for t in out["outs"] + [d for d in out["dacts"] if d is not None]:
        assert np.array_equal(t, orc.round_bf16(t))
    assert not np.array_equal(out["grads"][2]["w"], orc.round_bf16(out["grads"][2]["w"]))
    ref = orc.network_train_step(L, P, x, np.array([0, 3, 4, 1]), 0.1, 0.9)
    assert abs(out["loss"] - ref["loss"]) < 2e-2
