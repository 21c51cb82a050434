"""Parity of the HIP library (through its C ABI) against the CPU checker, element by element on the
same seeded inputs.  Tolerances: max relative error 1e-4 for fp32, 2e-2 for bf16 storage with fp32
accumulate; integer results (pooling argmax) bit-exact.

Relative error of a tensor: max_i |g_i - r_i| / max(|r_i|, rms(r)) -- the rms floor keeps the exact
zeros a ReLU produces from turning rounding noise into infinite relative error."""
import numpy as np
import pytest
import torch

import oracle as orc
from paper_2003_10688_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def sol():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2003_10688_amd import sol as s

    s.lib()
    return s


def rel_err(g, r):
    g, r = np.asarray(g, np.float64), np.asarray(r, np.float64)
    assert g.shape == r.shape, (g.shape, r.shape)
    if r.size == 0:
        return 0.0
    floor = max(np.sqrt(np.mean(r * r)), 1e-30)
    return float(np.max(np.abs(g - r) / np.maximum(np.abs(r), floor)))


def _dt(sol, name):
    return sol.BF16 if name == "bf16" else sol.F32


def _grid(a, name):
    return wl.to_bf16_grid(a) if name == "bf16" else np.asarray(a, np.float32)


def make_block(sol, rng, dt, N, C, H, W, K, k, s, p, bn=True, act="relu", pool=None, res=False, bias_std=0.3):
    l = wl.conv(K, k, s, p, bn=bn, act=act, pool=pool)
    x = _grid(rng.standard_normal((N, C, H, W)), dt)
    prm = {"w": _grid(rng.standard_normal((K, C, k, k)) * np.sqrt(2.0 / (C * k * k)), dt),
           "bias": (rng.standard_normal(K) * bias_std).astype(np.float32)}
    if bn:
        prm.update(gamma=rng.uniform(0.5, 1.5, K).astype(np.float32), beta=rng.uniform(-0.1, 0.1, K).astype(np.float32),
                   mean=(rng.standard_normal(K) * 0.1).astype(np.float32), var=rng.uniform(0.5, 1.5, K).astype(np.float32))
    Ho, Wo = orc.out_size(H, k, s, p), orc.out_size(W, k, s, p)
    r = _grid(rng.standard_normal((N, K, Ho, Wo)), dt) if res else None
    return l, x, prm, r


def run_block(sol, dt, l, x, prm, r, want_argmax=False, want_prepool=False):
    d = _dt(sol, dt)
    cd = sol.ConvDesc(l["cout"], x.shape[1], l["kh"], l["kw"], l["sh"], l["sw"], l["ph"], l["pw"])
    wp = sol.sol_pack_conv_weights(cd, d, sol.dev_f32(prm["w"]))
    bn = l["bn"]
    scale, shift = sol.sol_fold_bn(l["cout"], *(sol.dev_f32(prm[k]) if bn else None for k in ("gamma", "beta", "mean", "var")),
                                   sol.dev_f32(prm["bias"]), 1e-5)
    y, arg, pre = sol.sol_conv2d_fused(sol.to_device_nhwc(x, d), cd, wp, scale, shift,
                                       sol.to_device_nhwc(r, d) if r is not None else None,
                                       sol.ACT_RELU if l["act"] == "relu" else sol.ACT_NONE, l["pool"],
                                       want_argmax, want_prepool)
    torch.cuda.synchronize()
    return (sol.to_host_nchw(y), sol.to_host_nchw(arg) if arg is not None else None,
            sol.to_host_nchw(pre) if pre is not None else None)


CONV_CASES = [
    # N, C, H, W, K, k, s, p, res      several tiles + ragged tails in pixels and channels
    (2, 64, 19, 17, 96, 3, 1, 1, True),
    (3, 128, 14, 14, 80, 1, 1, 0, True),
    (2, 64, 23, 23, 64, 3, 2, 1, False),
    (1, 256, 9, 9, 520, 1, 2, 0, False),
    (2, 3, 37, 35, 64, 7, 2, 3, False),     # stem-like: Cin = 3 -> element gather path
    (2, 3, 37, 35, 32, 3, 2, 1, False),     # 3x3 stem of the separable chain (bf16: stem kernel, one 32-channel block)
    (1, 3, 64, 48, 64, 3, 2, 1, True),
    (2, 3, 20, 21, 24, 3, 2, 0, False),
    (2, 3, 33, 40, 24, 7, 2, 3, False),
    (5, 3, 16, 16, 16, 3, 1, 1, False),
    (1, 24, 11, 11, 40, 3, 1, 1, True),     # Cin not a multiple of the 128-byte chunk -> gather path
    (2, 32, 12, 12, 32, 5, 1, 2, False),
    (1, 64, 1, 1, 10, 1, 1, 0, False),      # degenerate 1x1 image, Cout not a multiple of 4
    (2, 64, 1, 1, 10, 1, 1, 1, True),       # ... with padding: 3x3 output pixels per image, eight of them act(shift + residual)
    (3, 32, 1, 1, 16, 1, 2, 2, False),      # ... padded and strided
    (130, 64, 2, 2, 64, 3, 1, 1, True),     # many tiny images
]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_fused_matches_oracle(sol, dt, case):
    N, C, H, W, K, k, s, p, res = case
    rng = np.random.default_rng(hash(case) % (2 ** 31))
    l, x, prm, r = make_block(sol, rng, dt, N, C, H, W, K, k, s, p, res=res)
    want, _, _ = orc.fused_conv(x, prm, l, r, bf16=(dt == "bf16"))
    got, _, _ = run_block(sol, dt, l, x, prm, r)
    assert rel_err(got, want) <= TOL[dt]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_conv_no_bn_no_act_plain(sol, dt):
    rng = np.random.default_rng(5)
    l, x, prm, r = make_block(sol, rng, dt, 2, 64, 10, 10, 64, 3, 1, 1, bn=False, act="none")
    want, _, _ = orc.fused_conv(x, prm, l, None, bf16=(dt == "bf16"))
    got, _, _ = run_block(sol, dt, l, x, prm, None)
    assert rel_err(got, want) <= TOL[dt]
    assert (got < 0).any()                       # really no ReLU


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_conv_weight_heavy_layer(sol, dt):
    """Weights larger than the input (and than 1.5 MB): the planner hands each XCD a set of channel tiles
    instead of a run of pixel tiles; every output element is compared."""
    rng = np.random.default_rng(77)
    l, x, prm, r = make_block(sol, rng, dt, 3, 512, 7, 7, 1024, 3, 1, 1, res=True)
    want, _, _ = orc.fused_conv(x, prm, l, r, bf16=(dt == "bf16"))
    got, _, _ = run_block(sol, dt, l, x, prm, r)
    assert rel_err(got, want) <= TOL[dt]


@pytest.mark.parametrize("tile", list(range(1, 9)) + list(range(11, 19)) + list(range(21, 28)) + [31, 32, 33])
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_every_conv_tile(sol, dt, tile):
    rng = np.random.default_rng(100 + tile)
    l, x, prm, r = make_block(sol, rng, dt, 2, 64, 21, 20, 136, 3, 1, 1, res=True)
    want, _, _ = orc.fused_conv(x, prm, l, r, bf16=(dt == "bf16"))
    sol.sol_debug_set_conv_tile(tile)
    try:
        got, _, _ = run_block(sol, dt, l, x, prm, r)
    finally:
        sol.sol_debug_set_conv_tile(0)
    assert rel_err(got, want) <= TOL[dt]



HALO_CASES = [
    # N, C, H, W, K, res     3x3 / stride 1 / pad 1: ragged pixel and channel tails, several input chunks,
    # tiles that span many images, image widths from 1 to 56
    (2, 64, 21, 20, 136, True),
    (3, 192, 14, 14, 256, False),
    (5, 512, 7, 7, 128, True),
    (130, 64, 2, 2, 64, True),
    (3, 128, 1, 1, 64, False),
    (2, 64, 5, 1, 72, False),
    (1, 128, 28, 28, 128, False),
    (2, 64, 33, 30, 64, True),
]


@pytest.mark.parametrize("tile", [41, 42, 43, 46, 47, 48, 49])
@pytest.mark.parametrize("case", HALO_CASES)
def test_halo_conv_tiles(sol, tile, case):
    """The 3x3 halo-in-LDS kernel in each of its tile shapes against the checker, every output element."""
    N, C, H, W, K, res = case
    rng = np.random.default_rng(hash((tile,) + case) % (2 ** 31))
    l, x, prm, r = make_block(sol, rng, "bf16", N, C, H, W, K, 3, 1, 1, res=res)
    want, _, _ = orc.fused_conv(x, prm, l, r, bf16=True)
    sol.sol_debug_set_conv_tile(tile)
    try:
        got, _, _ = run_block(sol, "bf16", l, x, prm, r)
    finally:
        sol.sol_debug_set_conv_tile(0)
    assert rel_err(got, want) <= TOL["bf16"]


@pytest.mark.parametrize("tile", [44, 45])
@pytest.mark.parametrize("case", [(1, 64, 56, 56, 64, False), (2, 64, 33, 50, 72, True), (3, 64, 9, 61, 64, False)])
def test_halo_conv_wide_single_chunk(sol, case, tile):
    """Wide images with one 64-channel input chunk (the first ResNet-50 stage) use the single-patch-buffer tile."""
    N, C, H, W, K, res = case
    rng = np.random.default_rng(hash(case) % (2 ** 31))
    l, x, prm, r = make_block(sol, rng, "bf16", N, C, H, W, K, 3, 1, 1, res=res)
    want, _, _ = orc.fused_conv(x, prm, l, r, bf16=True)
    sol.sol_debug_set_conv_tile(tile)
    try:
        got, _, _ = run_block(sol, "bf16", l, x, prm, r)
    finally:
        sol.sol_debug_set_conv_tile(0)
    assert rel_err(got, want) <= TOL["bf16"]


@pytest.mark.parametrize("case", [(1, 128, 56, 56, 32, False), (2, 192, 33, 50, 72, True), (3, 128, 9, 61, 64, False), (2, 64, 21, 20, 40, True),
                                  (1, 256, 40, 62, 32, False)])
def test_halo_conv_wide_several_chunks(sol, case):
    """Wide images (up to 62 columns) with several 64-channel input chunks and at most 64 output channels per tile -- the
    3x3 convolutions of a DenseNet-shaped first block -- on the tile with two patch buffers of 384 rows; plus an
    exact-integer run on it (bit for bit)."""
    N, C, H, W, K, res = case
    rng = np.random.default_rng(hash(case) % (2 ** 31))
    l, x, prm, r = make_block(sol, rng, "bf16", N, C, H, W, K, 3, 1, 1, res=res)
    want, _, _ = orc.fused_conv(x, prm, l, r, bf16=True)
    sol.sol_debug_set_conv_tile(50)
    try:
        got, _, _ = run_block(sol, "bf16", l, x, prm, r)
        assert rel_err(got, want) <= TOL["bf16"]
        xi = rng.integers(-2, 3, (N, C, H, W)).astype(np.float32)
        wi = (rng.integers(-1, 2, (K, C, 3, 3)) * (rng.random((K, C, 3, 3)) < 0.03)).astype(np.float32)
        li = wl.conv(K, 3, 1, 1, bn=False, act="none")
        pi = {"w": wi, "bias": np.zeros(K, np.float32)}
        wanti, _, _ = orc.fused_conv(xi, pi, li, None, bf16=True)
        assert np.abs(wanti).max() <= 256
        goti, _, _ = run_block(sol, "bf16", li, xi, pi, None)
        assert np.array_equal(goti, wanti)
    finally:
        sol.sol_debug_set_conv_tile(0)


def test_halo_conv_exact_integers(sol):
    """Small-integer inputs and weights: every product and partial sum is exact in fp32 and the outputs are exact
    in bf16, so the halo kernel must agree with the checker bit for bit (a wrong tap, border mask or patch row
    cannot hide inside the tolerance)."""
    rng = np.random.default_rng(11)
    N, C, H, W, K = 3, 128, 13, 11, 64
    x = rng.integers(-2, 3, (N, C, H, W)).astype(np.float32)
    w = (rng.integers(-1, 2, (K, C, 3, 3)) * (rng.random((K, C, 3, 3)) < 0.05)).astype(np.float32)
    l = wl.conv(K, 3, 1, 1, bn=False, act="none")
    prm = {"w": w, "bias": np.zeros(K, np.float32)}
    want, _, _ = orc.fused_conv(x, prm, l, None, bf16=True)
    assert np.abs(want).max() <= 256 and np.abs(want).max() > 4
    for tile in (41, 42, 43, 46, 47, 48):
        sol.sol_debug_set_conv_tile(tile)
        try:
            got, _, _ = run_block(sol, "bf16", l, x, prm, None)
        finally:
            sol.sol_debug_set_conv_tile(0)
        assert np.array_equal(got, want), tile


GEMM8_CASES = [
    # N, C, H, W, K, k, stride, res, pool     ragged tails, long and short reductions, stride 2, filter taps with padding, fused pool
    (2, 64, 21, 20, 136, 1, 1, True, None),
    (3, 256, 14, 14, 520, 1, 2, False, None),
    (5, 2048, 7, 7, 512, 1, 1, False, None),
    (2, 1024, 7, 7, 264, 1, 1, True, None),
    (1, 32, 9, 9, 40, 1, 1, False, None),
    (2, 64, 16, 16, 64, 1, 1, False, "max"),
    (70, 128, 3, 3, 128, 1, 1, True, None),
    (3, 128, 15, 14, 136, 3, 2, False, None),
    (2, 64, 23, 23, 64, 3, 1, True, None),
    (2, 64, 12, 12, 72, 5, 2, False, None),
    (40, 512, 2, 2, 64, 3, 2, False, None),
]


@pytest.mark.parametrize("tile", list(range(61, 71)))
@pytest.mark.parametrize("case", GEMM8_CASES)
def test_gemm8_conv_tiles(sol, tile, case):
    """The eight-wave implicit-GEMM kernel in each tile shape (with and without the in-workgroup K split) against the
    checker, every output element."""
    N, C, H, W, K, k, st, res, pool = case
    if C % 64 and tile not in (66, 67):
        pytest.skip("128-byte-row tiles need Cin % 64 == 0")
    if C % 128 and tile == 70:
        pytest.skip("the 256-byte-row tile needs Cin % 128 == 0")
    rng = np.random.default_rng(hash((tile,) + case) % (2 ** 31))
    pd = dict(kind=pool, kh=2, kw=2, sh=2, sw=2, ph=0, pw=0) if pool else None
    l, x, prm, r = make_block(sol, rng, "bf16", N, C, H, W, K, k, st, k // 2, res=res, pool=pd)
    want, _, _ = orc.fused_conv(x, prm, l, r, bf16=True)
    sol.sol_debug_set_conv_tile(tile)
    try:
        got, _, _ = run_block(sol, "bf16", l, x, prm, r)
    finally:
        sol.sol_debug_set_conv_tile(0)
    assert rel_err(got, want) <= TOL["bf16"]


def test_gemm8_conv_exact_integers(sol):
    """Small-integer operands make every partial sum exact in fp32, so all tile shapes (any split of the
    reduction) must reproduce the checker bit for bit."""
    rng = np.random.default_rng(12)
    N, C, H, W, K = 3, 512, 9, 7, 192
    x = rng.integers(-2, 3, (N, C, H, W)).astype(np.float32)
    w = (rng.integers(-1, 2, (K, C, 1, 1)) * (rng.random((K, C, 1, 1)) < 0.1)).astype(np.float32)
    l = wl.conv(K, 1, 1, 0, bn=False, act="none")
    prm = {"w": w, "bias": np.zeros(K, np.float32)}
    want, _, _ = orc.fused_conv(x, prm, l, None, bf16=True)
    assert 4 < np.abs(want).max() <= 256
    for tile in range(61, 71):
        sol.sol_debug_set_conv_tile(tile)
        try:
            got, _, _ = run_block(sol, "bf16", l, x, prm, None)
        finally:
            sol.sol_debug_set_conv_tile(0)
        assert np.array_equal(got, want), tile

@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("kind", ["max", "avg"])
@pytest.mark.parametrize("shape", [(2, 3, 32, 32, 16), (3, 64, 15, 13, 72), (1, 32, 8, 8, 64)])
def test_fused_pool_values(sol, dt, kind, shape):
    """Random data: pooled values within tolerance; every argmax points into its own window at an
    element whose pre-pool value equals the window maximum up to the tolerance."""
    N, C, H, W, K = shape
    rng = np.random.default_rng(11)
    l, x, prm, _ = make_block(sol, rng, dt, N, C, H, W, K, 3, 1, 1, pool=wl.pool_desc(kind, 2, 2, 0))
    want, warg, wpre = orc.fused_conv(x, prm, l, None, bf16=(dt == "bf16"), want_prepool=True)
    got, garg, gpre = run_block(sol, dt, l, x, prm, None, want_argmax=(kind == "max"), want_prepool=True)
    assert got.shape == (N, K, H // 2, W // 2)
    assert rel_err(got, want) <= TOL[dt]
    wpre_st = orc.round_bf16(wpre) if dt == "bf16" else wpre
    assert rel_err(gpre[:, :, :H // 2 * 2, :W // 2 * 2], wpre_st[:, :, :H // 2 * 2, :W // 2 * 2]) <= TOL[dt]
    if kind == "max":
        ih, iw = garg // W, garg % W
        pp, qq = np.meshgrid(np.arange(H // 2), np.arange(W // 2), indexing="ij")
        assert np.all((ih // 2 == pp) & (iw // 2 == qq))
        picked = np.take_along_axis(wpre.reshape(N, K, -1), garg.reshape(N, K, -1).astype(np.int64), 2).reshape(want.shape)
        wmax = orc.maxpool(wpre, (2, 2), (2, 2), (0, 0))[0]
        floor = np.sqrt(np.mean(wmax * wmax))
        assert np.max(np.abs(picked - wmax) / np.maximum(np.abs(wmax), floor)) <= TOL[dt]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_fused_pool_argmax_bit_exact(sol, dt):
    """Small-integer inputs, weights and affine map: every intermediate is exact in fp32, so the HIP
    path and the checker see identical pre-pool values, full of exact ties (ReLU zeros and integer
    collisions).  Values and argmax must then agree bit for bit (first maximum in window order wins)."""
    rng = np.random.default_rng(3)
    N, C, H, W, K = 2, 32, 14, 18, 48
    l = wl.conv(K, 3, 1, 1, bn=False, act="relu", pool=wl.pool_desc("max", 2, 2, 0))
    x = rng.integers(-2, 3, (N, C, H, W)).astype(np.float32)
    prm = {"w": rng.integers(-1, 2, (K, C, 3, 3)).astype(np.float32), "bias": rng.integers(-3, 4, K).astype(np.float32)}
    want, warg, wpre = orc.fused_conv(x, prm, l, None, bf16=False, want_prepool=True)
    assert np.abs(wpre).max() <= 256 and (wpre == 0).mean() > 0.3          # exact in bf16 too; many ties
    got, garg, gpre = run_block(sol, dt, l, x, prm, None, want_argmax=True, want_prepool=True)
    assert np.array_equal(gpre, wpre)
    assert np.array_equal(got, want)
    assert np.array_equal(garg, warg)


POOL_CASES = [("max", 3, 2, 1), ("max", 2, 2, 0), ("max", 3, 1, 1), ("avg", 3, 2, 1), ("avg", 2, 2, 0), ("max", 5, 3, 2)]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("cfg", POOL_CASES)
@pytest.mark.parametrize("shape", [(2, 64, 29, 31), (1, 20, 9, 9), (3, 7, 6, 5)])
def test_pool_matches_oracle(sol, dt, cfg, shape):
    kind, k, s, p = cfg
    rng = np.random.default_rng(17)
    x = _grid(np.round(rng.standard_normal(shape) * 4) / 4, dt)            # coarse grid: many exact ties
    d = _dt(sol, dt)
    for cp in ((1, 0) if kind == "avg" else (1,)):
        pd = wl.pool_desc(kind, k, s, p, cp)
        y, arg = sol.sol_pool(sol.to_device_nhwc(x, d), pd, want_argmax=(kind == "max"))
        torch.cuda.synchronize()
        want, warg = orc.pool(x, pd)
        if kind == "max":
            assert np.array_equal(sol.to_host_nchw(y), want)               # selection only: exact
            assert np.array_equal(sol.to_host_nchw(arg), warg)             # integer result: bit-exact
        else:
            want = orc.round_bf16(want) if dt == "bf16" else want
            assert rel_err(sol.to_host_nchw(y), want) <= TOL[dt]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(64, 2048, 7, 7), (3, 64, 8, 8), (2, 10, 5, 3), (1, 8, 1, 1)])
def test_global_avgpool(sol, dt, shape):
    rng = np.random.default_rng(23)
    x = _grid(rng.standard_normal(shape) + 0.5, dt)
    y = sol.sol_global_avgpool(sol.to_device_nhwc(x, _dt(sol, dt)))
    torch.cuda.synchronize()
    want = orc.gap(x)
    want = orc.round_bf16(want) if dt == "bf16" else want
    assert rel_err(sol.to_host_nchw(y)[:, :, 0, 0], want) <= TOL[dt]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(64, 2048, 1000), (64, 64, 10), (5, 100, 33), (1, 7, 3), (130, 512, 1000), (200, 96, 40),
                                   (1100, 64, 8), (32, 1000, 512), (9, 24, 16),      # the last two: rows end in half an MFMA step
                                   (3, 8, 5), (33, 16, 31), (64, 8200, 40)])         # one fragment per row; rounds that run past the end
def test_linear(sol, dt, shape):
    M, I, O = shape
    rng = np.random.default_rng(29)
    d = _dt(sol, dt)
    x = _grid(rng.standard_normal((M, I)), dt)
    w = _grid(rng.standard_normal((O, I)) * np.sqrt(2.0 / I), dt)
    b = rng.standard_normal(O).astype(np.float32)
    cd = sol.ConvDesc(O, I, 1, 1, 1, 1, 0, 0)
    wp = sol.sol_pack_conv_weights(cd, d, sol.dev_f32(w.reshape(O, I, 1, 1)))
    for act in ("none", "relu"):
        y = sol.sol_linear(sol.to_device_nhwc(x, d), wp, sol.dev_f32(b), O, sol.ACT_RELU if act == "relu" else sol.ACT_NONE)
        torch.cuda.synchronize()
        want = orc.linear(x, w, b)
        want = orc.relu(want) if act == "relu" else want
        want = orc.round_bf16(want) if dt == "bf16" else want
        assert rel_err(sol.to_host_nchw(y), want) <= TOL[dt]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_pack_unpack_roundtrip(sol, dt):
    rng = np.random.default_rng(31)
    for (K, C, R, S) in [(16, 3, 3, 3), (64, 64, 3, 3), (10, 7, 1, 1), (64, 3, 7, 7)]:
        w = _grid(rng.standard_normal((K, C, R, S)), dt)
        cd = sol.ConvDesc(K, C, R, S, 1, 1, 0, 0)
        wp = sol.sol_pack_conv_weights(cd, _dt(sol, dt), sol.dev_f32(w))
        back = sol.sol_unpack_conv_weights(cd, _dt(sol, dt), wp)
        torch.cuda.synchronize()
        assert np.array_equal(back.cpu().numpy(), w)


def test_bf16_store_rounding_is_nearest_even(sol):
    """Every fp32 -> bf16 store of the HIP path uses one conversion; check it bit for bit against the
    checker's rounding on random magnitudes, exact ties, values next to ties, and tiny/huge values."""
    rng = np.random.default_rng(37)
    v = (rng.standard_normal(60000) * np.exp(rng.uniform(-30, 30, 60000))).astype(np.float32)
    base = (rng.standard_normal(2000) * np.exp(rng.uniform(-10, 10, 2000))).astype(np.float32)
    grid = wl.to_bf16_grid(base).view(np.uint32)
    ties = (grid | 0x8000).view(np.float32)                      # exactly half way to the next bf16 value
    near = np.concatenate([(grid | 0x8001).view(np.float32), (grid | 0x7fff).view(np.float32)])
    w = np.concatenate([v, ties, near, np.float32([0.0, -0.0, 1e-40, -1e-40, 3.38e38, 1.0, -1.0])])
    w = np.resize(w, (64, 1024 // 1, 1, 1)).astype(np.float32)
    cd = sol.ConvDesc(64, 1024, 1, 1, 1, 1, 0, 0)
    back = sol.sol_unpack_conv_weights(cd, sol.BF16, sol.sol_pack_conv_weights(cd, sol.BF16, sol.dev_f32(w)))
    torch.cuda.synchronize()
    assert np.array_equal(back.cpu().numpy().astype(np.float64), orc.round_bf16(w.astype(np.float64)))


def test_empty_batch_and_errors(sol):
    d = sol.F32
    cd = sol.ConvDesc(8, 4, 3, 3, 1, 1, 1, 1)
    wp = sol.sol_pack_conv_weights(cd, d, sol.dev_f32(np.zeros((8, 4, 3, 3), np.float32)))
    x0 = torch.empty((0, 5, 5, 4), device="cuda:0")
    y, _, _ = sol.sol_conv2d_fused(x0, cd, wp)
    assert y.shape == (0, 5, 5, 8)
    y, _ = sol.sol_pool(x0, wl.pool_desc("max", 2, 2, 0))
    assert y.shape == (0, 2, 2, 4)
    x = torch.zeros((1, 5, 5, 4), device="cuda:0")
    with pytest.raises(sol.SolError) as e:
        sol.sol_conv2d_fused(x, cd, wp, pool=wl.pool_desc("max", 3, 2, 1))
    assert e.value.status == 6
    with pytest.raises(sol.SolError) as e:
        sol.sol_conv2d_fused(torch.zeros((1, 5, 5, 3), device="cuda:0"), cd, wp)
    assert e.value.status == 2
    with pytest.raises(sol.SolError) as e:                                   # misaligned pointer
        sol.sol_conv2d_fused(torch.zeros(101, device="cuda:0")[1:].view(1, 5, 5, 4), cd, wp)
    assert e.value.status == 4


def test_network_on_an_empty_batch(sol):
    """A network planned for batch 0 (concatenation, fused stem pair and projection pair included) accepts the NULL
    pointers an allocator hands out for empty tensors and launches nothing, like the single-layer calls."""
    c = wl.conv
    layers = [c(64, 7, s=2, p=3), wl.pool("max", 3, 2, 1), c(64, 1, p=0), c(64, 3), c(256, 1, p=0, act="none", src=1),
              c(256, 1, p=0, src=3, res=4), c(32, 1, p=0, bn=False, src=5), c(32, 3, bn=False, src=5), wl.concat(6, 7), wl.gap(),
              wl.linear(10)]
    for flags in (0, sol.NET_KEEP_ACTIVATIONS):
        net = sol.Network(layers, (0, 3, 64, 64), sol.BF16, flags=flags)
        net.set_params(wl.make_params(layers, 3, 1, True))
        x0 = torch.empty((0, 64, 64, 3), dtype=torch.bfloat16, device="cuda:0")
        assert x0.data_ptr() == 0 or x0.numel() == 0
        y = net.forward(x0)
        torch.cuda.synchronize()
        assert tuple(y.shape) == (0, 1, 1, 10)
        assert net.autotune(x0, reps=1) == {}
        assert tuple(net.forward_static(x0).shape) == (0, 1, 1, 10)


def test_nan_propagates_alike_through_both_epilogues(sol):
    """A NaN in the input reaches every output it feeds as NaN when no activation follows, in interior tiles (fast
    epilogue) and in ragged edge tiles (general epilogue) alike; behind a ReLU both store 0 (v > 0 is false for NaN)."""
    rng = np.random.default_rng(2)
    for dt in ("f32", "bf16"):
        for act, cout in (("none", 64), ("relu", 64), ("none", 72)):
            l, x, prm, _ = make_block(sol, rng, dt, 2, 64, 13, 11, cout, 1, 1, 0, bn=True, act=act)
            x[:, 5] = np.nan                       # one input channel: every output pixel sees it
            got, _, _ = run_block(sol, dt, l, x, prm, None)
            if act == "none":
                assert np.isnan(got).all(), (dt, act, cout, np.count_nonzero(~np.isnan(got)))
            else:
                assert (got == 0).all(), (dt, act, cout)


# ---------------------------------------------------------------------------------- whole networks
def run_network(sol, wk, keep=True):
    d = _dt(sol, wk.dtype)
    net = sol.Network(wk.layers, wk.in_shape, d, flags=sol.NET_KEEP_ACTIVATIONS if keep else 0)
    net.set_params(wk.params)
    y = net.forward(sol.to_device_nhwc(wk.x, d))
    torch.cuda.synchronize()
    return net, sol.to_host_nchw(y)


def _layer_results(sol, net, y, outs):
    got = [sol.to_host_nchw(net.layer_output(i)).reshape(outs[i].shape) for i in range(len(outs) - 1)]
    got.append(y.reshape(outs[-1].shape))
    return got


def norm_err(g, r):
    return float(np.linalg.norm(np.asarray(g, np.float64) - r) / max(np.linalg.norm(r), 1e-30))


@pytest.mark.parametrize("cfg,batch,hw", [(0, None, None), (1, None, None), (1, 5, 18)])
def test_network_forward_fp32_configs(sol, cfg, batch, hw):
    """Configs 0 and 1 end to end at their full size; every layer's stored output is compared."""
    wk = wl.config(cfg, batch=batch, hw=hw)
    outs, _ = orc.network_forward(wk.layers, wk.params, wk.x, return_all=True)
    net, y = run_network(sol, wk)
    errs = [rel_err(g, r) for g, r in zip(_layer_results(sol, net, y, outs), outs)]
    print(f"cfg{cfg} per-layer rel err: max {max(errs):.3e} last {errs[-1]:.3e}")
    assert max(errs) <= TOL["f32"], errs
    _, y2 = run_network(sol, wk, keep=False)          # the buffer-reusing plan gives the same result
    assert np.array_equal(y, y2)


@pytest.mark.parametrize("cfg,batch,hw", [(2, 2, 64), (3, 2, 64), (3, 1, 224), (6, 3, 64), (6, 1, 224)])
def test_network_forward_resnets_fp32_arithmetic(sol, cfg, batch, hw):
    """The ResNet-shaped layer lists in fp32 storage: no rounding points between layers, so the whole
    chain (planner wiring, residual edges, every kernel template) must agree to 1e-4 end to end."""
    wk = wl.config(cfg, batch=batch, hw=hw, dtype="f32")
    outs, _ = orc.network_forward(wk.layers, wk.params, wk.x, return_all=True)
    net, y = run_network(sol, wk)
    errs = [rel_err(g, r) for g, r in zip(_layer_results(sol, net, y, outs), outs)]
    print(f"cfg{cfg}/fp32 per-layer rel err: max {max(errs):.3e} last {errs[-1]:.3e}")
    assert max(errs) <= TOL["f32"], errs


@pytest.mark.parametrize("cfg,batch,hw", [(2, 2, 64), (3, 2, 64), (3, 1, 224), (2, 1, 224), (6, 3, 64), (6, 1, 224)])
def test_network_forward_resnets_bf16(sol, cfg, batch, hw):
    """bf16 storage, fp32 accumulate.  Two passes over the same seeded tensors:

    (a) layer by layer inside the network object: every layer consumes the CHECKER's stored
        activations (exact bf16 values) and its output must match element-wise within 2e-2;
    (b) free running: the network consumes its own activations.  A bf16 store that rounds the other
        way than the checker's (fp32 vs fp64 accumulation straddling a rounding boundary) perturbs the
        next layer's sums, which flips more roundings; over 20-50 layers the element-wise maximum
        over ~10^6 values drifts to several bf16 ulps although the typical element stays within one.
        So (b) is gated on the norm-wise relative error (2e-2) at every layer and a loose element-wise
        bound; the strict element-wise statement is (a)."""
    wk = wl.config(cfg, batch=batch, hw=hw)
    outs, _ = orc.network_forward(wk.layers, wk.params, wk.x, bf16=True, return_all=True)
    net, y = run_network(sol, wk)
    free = _layer_results(sol, net, y, outs)
    e_free = [rel_err(g, r) for g, r in zip(free, outs)]
    n_free = [norm_err(g, r) for g, r in zip(free, outs)]
    # (a) teacher-forced: load the checker's activations into the workspace, run one layer at a time
    nl = len(wk.layers)
    x = sol.to_device_nhwc(wk.x, sol.BF16)
    dev = [sol.to_device_nhwc(o if o.ndim == 4 else o[:, :, None, None], sol.BF16) for o in outs]
    for i in range(nl - 1):
        net.layer_output(i).copy_(dev[i])
    e_forced = []
    for i in range(nl):
        net.run_layer(i, x)
        torch.cuda.synchronize()
        g = sol.to_host_nchw(net.y if i == nl - 1 else net.layer_output(i)).reshape(outs[i].shape)
        e_forced.append(rel_err(g, outs[i]))
        if i < nl - 1:
            net.layer_output(i).copy_(dev[i])
    print(f"cfg{cfg} bf16 b{batch} hw{hw}: layer-by-layer max {max(e_forced):.3e} | free-running element-wise max "
          f"{max(e_free):.3e} last {e_free[-1]:.3e}, norm-wise max {max(n_free):.3e}")
    assert max(e_forced) <= TOL["bf16"], e_forced
    assert max(n_free) <= TOL["bf16"], n_free
    assert max(e_free) <= 0.25, e_free
    _, y2 = run_network(sol, wk, keep=False)
    # the lean plan fuses layer pairs; a projection shortcut computed inside the launch that adds it is not rounded to
    # bf16 on the way (the kept-activation plan stores it), so the two plans agree within the tolerance, not bit for bit
    assert norm_err(y2, y.astype(np.float64)) <= TOL["bf16"]
    assert norm_err(y2.reshape(outs[-1].shape), outs[-1]) <= TOL["bf16"]


def test_network_deterministic(sol):
    wk = wl.config(2, batch=2, hw=64)
    _, y1 = run_network(sol, wk, keep=False)
    _, y2 = run_network(sol, wk, keep=False)
    assert np.array_equal(y1, y2)


def _distinct_conv_shapes(wk):
    """(layer index, input shape NCHW) of one representative per distinct convolution geometry."""
    n, c, h, w = wk.in_shape
    shapes, seen, out = [], {}, []
    for i, l in enumerate(wk.layers):
        s = l.get("src", -1)
        ins = (n, c, h, w) if (i == 0 and s == -1) else shapes[i - 1 if s == -1 else s]
        if l["kind"] == "conv":
            o = (ins[0], l["cout"], orc.out_size(ins[2], l["kh"], l["sh"], l["ph"]), orc.out_size(ins[3], l["kw"], l["sw"], l["pw"]))
            key = (ins, l["cout"], l["kh"], l["sh"], l["res"] >= 0, l["act"])
            if key not in seen:
                seen[key] = i
                out.append((i, ins))
        elif l["kind"] == "pool":
            pd = l["pool"]
            o = (ins[0], ins[1], orc.out_size(ins[2], pd["kh"], pd["sh"], pd["ph"]), orc.out_size(ins[3], pd["kw"], pd["sw"], pd["pw"]))
        elif l["kind"] == "gap":
            o = (ins[0], ins[1], 1, 1)
        else:
            o = (ins[0], l["out"], 1, 1)
        shapes.append(o)
    return out


@pytest.mark.parametrize("cfg", [3, 2])
def test_full_size_layers_sampled(sol, cfg):
    """Every distinct convolution geometry of the ResNet-shaped configs at the full benchmark batch,
    in the automatically planned launch configuration, on seeded synthetic inputs; 256 sampled outputs
    per layer are recomputed one by one by the checker."""
    wk = wl.config(cfg)
    d = _dt(sol, wk.dtype)
    rng = np.random.default_rng(wk.seed)
    worst = 0.0
    for i, ins in _distinct_conv_shapes(wk):
        l, prm = wk.layers[i], wk.params[i]
        x = wl.to_bf16_grid(rng.standard_normal(ins, dtype=np.float32))
        K = l["cout"]
        Ho, Wo = orc.out_size(ins[2], l["kh"], l["sh"], l["ph"]), orc.out_size(ins[3], l["kw"], l["sw"], l["pw"])
        r = wl.to_bf16_grid(rng.standard_normal((ins[0], K, Ho, Wo), dtype=np.float32)) if l["res"] >= 0 else None
        got, _, _ = run_block(sol, wk.dtype, dict(l, pool=None), x, prm, r)
        coords = np.stack([rng.integers(0, s, 256) for s in (ins[0], K, Ho, Wo)], 1)
        coords[:8] = [[0, 0, 0, 0], [ins[0] - 1, K - 1, Ho - 1, Wo - 1], [0, K - 1, 0, Wo - 1], [ins[0] - 1, 0, Ho - 1, 0],
                      [0, 0, Ho - 1, Wo - 1], [ins[0] - 1, K - 1, 0, 0], [ins[0] // 2, K // 2, Ho // 2, Wo // 2], [0, 1, 0, 1]]
        want = orc.fused_conv_points(x, prm, dict(l, pool=None), coords, r, bf16=True)
        g = got[tuple(coords.T)]
        floor = np.sqrt(np.mean(want * want)) + 1e-30
        err = float(np.max(np.abs(g - want) / np.maximum(np.abs(want), floor)))
        worst = max(worst, err)
        print(f"  L{i} in{ins} k{l['kh']} s{l['sh']} cout{K}: rel err {err:.3e} ({np.count_nonzero(g != want)} of {len(g)} differ)", flush=True)
        assert err <= TOL["bf16"], (i, ins, l, err)
        del x, got, r
    print(f"cfg{cfg} full-size sampled layers: worst rel err {worst:.3e}")


def test_full_size_projection_pairs_in_the_tuned_plan(sol):
    """The four projection-pair launches of the ResNet-50-shaped pass at batch 64, inside the lean network object and
    after the plan-time auto-tune (the launch configuration bench.py times): both input tensors of a pair are
    overwritten with seeded values, the pair layer is run alone, and 256 sampled outputs are recomputed by the checker
    from both convolutions.  Strict statement: against the checker's pieces with the shortcut left unrounded, as the
    kernel computes it (2e-2); the checker's own definition, which stores -- and so rounds -- the shortcut, within
    twice that.  The other layers of the tuned plan are covered by the sampled checks above and by bench.py's own
    comparison of the timed output with the checker."""
    wk = wl.config(3)
    net = sol.Network(wk.layers, wk.in_shape, sol.BF16)              # lean plan: pairs fused, buffers reused
    net.set_params(wk.params)
    x = sol.to_device_nhwc(wk.x, sol.BF16)
    net.autotune(x, reps=2)
    net.forward(x)
    torch.cuda.synchronize()
    L, P = wk.layers, wk.params
    ins, outs = {}, {}
    shp = wk.in_shape
    for i, l in enumerate(L):                                        # logical shapes, by bookkeeping only
        s = l.get("src", -1)
        xin = shp if (i == 0 and s == -1) else outs[i - 1 if s == -1 else s]
        ins[i] = xin
        if l["kind"] == "conv":
            outs[i] = (xin[0], l["cout"], orc.out_size(xin[2], l["kh"], l["sh"], l["ph"]), orc.out_size(xin[3], l["kw"], l["sw"], l["pw"]))
        elif l["kind"] == "pool":
            pd = l["pool"]
            outs[i] = (xin[0], xin[1], orc.out_size(xin[2], pd["kh"], pd["sh"], pd["ph"]), orc.out_size(xin[3], pd["kw"], pd["sw"], pd["pw"]))
        elif l["kind"] == "gap":
            outs[i] = (xin[0], xin[1], 1, 1)
        else:
            outs[i] = (xin[0], l["out"], 1, 1)
    pairs = [(j, net.fused_into(j)) for j in range(len(L)) if L[j]["kind"] == "conv" and net.fused_into(j) != j]
    pairs = [(j, i) for j, i in pairs if L[i]["res"] == j]              # projection shortcuts (not the members of fused bottlenecks)
    assert len(pairs) == 4, pairs
    rng = np.random.default_rng(wk.seed + 9)
    src_of = lambda i: (i - 1) if L[i].get("src", -1) == -1 else L[i]["src"]   # noqa: E731
    for j, i in pairs:
        assert L[i]["res"] == j and L[j]["kh"] == 1 and L[i]["kh"] == 1
        xm = wl.to_bf16_grid(rng.standard_normal(ins[i], dtype=np.float32))     # input of the main 1x1 convolution
        xp = wl.to_bf16_grid(rng.standard_normal(ins[j], dtype=np.float32))     # block input, read by the shortcut
        net.layer_output(src_of(i)).copy_(sol.to_device_nhwc(xm, sol.BF16))
        net.layer_output(src_of(j)).copy_(sol.to_device_nhwc(xp, sol.BF16))
        net.run_layer(i, x)
        torch.cuda.synchronize()
        got = sol.to_host_nchw(net.layer_output(i))
        N, K, Ho, Wo = outs[i]
        assert got.shape == (N, K, Ho, Wo)
        coords = np.stack([rng.integers(0, s, 256) for s in (N, K, Ho, Wo)], 1).astype(np.int32)
        coords[:4] = [[0, 0, 0, 0], [N - 1, K - 1, Ho - 1, Wo - 1], [0, K - 1, 0, Wo - 1], [N - 1, 0, Ho - 1, 0]]
        lj, li = dict(L[j], pool=None), dict(L[i], pool=None)
        short = orc.fused_conv_points(xp, P[j], lj, coords, None, bf16=False)                       # conv + BN, no ReLU, unrounded
        main = orc.fused_conv_points(xm, P[i], dict(li, act="none"), coords, None, bf16=False)      # conv + BN of the main branch
        strict = orc.round_bf16(orc.relu(orc.add(main, short)))
        stored = orc.round_bf16(orc.relu(orc.add(main, orc.round_bf16(short))))                     # the checker's definition: the shortcut is a stored tensor
        g = got[tuple(coords.T)]
        floor = np.sqrt(np.mean(strict * strict)) + 1e-30
        e_strict = float(np.max(np.abs(g - strict) / np.maximum(np.abs(strict), floor)))
        e_stored = float(np.max(np.abs(g - stored) / np.maximum(np.abs(stored), floor)))
        print(f"  pair L{j}+L{i} in{ins[i]}/{ins[j]} -> {outs[i]}: strict {e_strict:.3e}, against the stored-shortcut definition {e_stored:.3e}", flush=True)
        assert e_strict <= TOL["bf16"], (j, i, e_strict)
        assert e_stored <= 2 * TOL["bf16"], (j, i, e_stored)


def test_full_size_fused_stem_pair_sampled(sol):
    """The depth-first stem + max-pool kernel at the benchmark's size (64 x 3 x 224 x 224, the launch the timed pass
    makes): sampled pooled outputs against the checker, each from the (up to) nine convolution points under its
    window -- convolution, explicit BN, ReLU, bf16 rounding, maximum."""
    wk = wl.config(3)
    l, prm = wk.layers[0], wk.params[0]
    pd = wk.layers[1]["pool"]
    assert (l["kh"], l["sh"], pd["kh"], pd["sh"], pd["ph"]) == (7, 2, 3, 2, 1)
    rng = np.random.default_rng(wk.seed + 5)
    x = wl.to_bf16_grid(rng.standard_normal(wk.in_shape, dtype=np.float32))
    got, _, _ = run_block(sol, "bf16", dict(l, pool=pd), x, prm, None)
    N, K, Ho, Wo = wk.in_shape[0], l["cout"], 112, 112
    Hy, Wy = got.shape[2], got.shape[3]
    assert got.shape == (N, K, 56, 56)
    pts = np.stack([rng.integers(0, s, 192) for s in (N, K, Hy, Wy)], 1)
    pts[:6] = [[0, 0, 0, 0], [N - 1, K - 1, Hy - 1, Wy - 1], [0, K - 1, 0, Wy - 1], [N - 1, 0, Hy - 1, 0], [N // 2, 31, 6, 7], [1, 32, 7, 8]]
    coords, owner = [], []
    for j, (n, k, py, px) in enumerate(pts):
        for dy in range(3):
            for dx in range(3):
                q, p = 2 * py - 1 + dy, 2 * px - 1 + dx
                if 0 <= q < Ho and 0 <= p < Wo:
                    coords.append((n, k, q, p)); owner.append(j)
    vals = orc.fused_conv_points(x, prm, dict(l, pool=None), np.array(coords), None, bf16=True)
    want = np.full(len(pts), -np.inf)
    np.maximum.at(want, np.array(owner), vals)
    g = got[tuple(pts.T)]
    floor = np.sqrt(np.mean(want * want)) + 1e-30
    err = float(np.max(np.abs(g - want) / np.maximum(np.abs(want), floor)))
    print(f"fused stem pair, full size: rel err {err:.3e} ({np.count_nonzero(g != want)} of {len(g)} differ)")
    assert err <= TOL["bf16"]


def test_full_size_stem_pool_and_gap(sol):
    wk = wl.config(3)
    rng = np.random.default_rng(1)
    x = wl.to_bf16_grid(rng.standard_normal((64, 64, 112, 112), dtype=np.float32))
    y, arg = sol.sol_pool(sol.to_device_nhwc(x, sol.BF16), wl.pool_desc("max", 3, 2, 1), want_argmax=True)
    torch.cuda.synchronize()
    y, arg = sol.to_host_nchw(y), sol.to_host_nchw(arg)
    for n in (0, 37, 63):                                                   # whole images, exact
        want, warg = orc.maxpool(x[n:n + 1], (3, 3), (2, 2), (1, 1))
        assert np.array_equal(y[n:n + 1], want) and np.array_equal(arg[n:n + 1], warg)


@pytest.mark.parametrize("cfg,batch,hw", [(1, 8, 32), (3, 2, 64), (7, 2, 64)])
def test_network_graph_replays(sol, cfg, batch, hw):
    """A recorded forward pass, replayed several times with new input contents and eager work and
    synchronisations between the replays, gives bit-identical results to the eager pass every time."""
    wk = wl.config(cfg, batch=batch, hw=hw)
    d = _dt(sol, wk.dtype)
    net = sol.Network(wk.layers, wk.in_shape, d)
    net.set_params(wk.params)
    x = sol.to_device_nhwc(wk.x, d)
    side = torch.cuda.Stream()
    launch = net.graph(x, side)
    rng = np.random.default_rng(3)
    for it in range(4):
        xi = _grid(rng.standard_normal(wk.in_shape), wk.dtype)
        x.copy_(sol.to_device_nhwc(xi, d))
        torch.cuda.synchronize()
        eager = net.forward(x).clone()                     # eager pass on the current stream
        torch.cuda.synchronize()
        net.y.zero_()
        junk = (torch.randn(1 << 16, device="cuda:0") * 2).sum()   # unrelated eager work between replays
        torch.cuda.synchronize()
        y = launch()
        side.synchronize()
        assert torch.equal(y, eager), f"replay {it} differs from the eager pass"
        assert bool((y.float().abs().sum() > 0).item())
        del junk
    with pytest.raises(sol.SolError) as e:                       # the NULL stream cannot be captured
        class _Null:
            cuda_stream = 0
        net.graph(x, _Null())
    assert e.value.status == 6


def test_network_autotune_keeps_results(sol):
    """Plan-time auto-tune: whatever kernels it picks, every layer still matches the checker (layer by layer on the
    checker's activations, element-wise) and a second pass reproduces the first bit for bit."""
    wk = wl.config(3, batch=2, hw=64)
    outs, _ = orc.network_forward(wk.layers, wk.params, wk.x, bf16=True, return_all=True)
    net = sol.Network(wk.layers, wk.in_shape, sol.BF16, flags=sol.NET_KEEP_ACTIVATIONS)
    net.set_params(wk.params)
    x = sol.to_device_nhwc(wk.x, sol.BF16)
    tuned = net.autotune(x, reps=3)
    assert all(0 < t < 100 for k, t in tuned.items() if not str(k).endswith("b"))
    y1 = sol.to_host_nchw(net.forward(x)).copy()
    y2 = sol.to_host_nchw(net.forward(x)).copy()
    assert np.array_equal(y1, y2)
    assert norm_err(y1.reshape(outs[-1].shape), outs[-1]) <= TOL["bf16"]
    nl = len(wk.layers)
    dev = [sol.to_device_nhwc(o if o.ndim == 4 else o[:, :, None, None], sol.BF16) for o in outs]
    for i in range(nl - 1):
        net.layer_output(i).copy_(dev[i])
    errs = []
    for i in range(nl):
        net.run_layer(i, x)
        torch.cuda.synchronize()
        g = sol.to_host_nchw(net.y if i == nl - 1 else net.layer_output(i)).reshape(outs[i].shape)
        errs.append(rel_err(g, outs[i]))
        if i < nl - 1:
            net.layer_output(i).copy_(dev[i])
    print(f"autotuned layers {tuned}; layer-by-layer max rel err {max(errs):.3e}")
    assert max(errs) <= TOL["bf16"], errs


@pytest.mark.parametrize("batch,features", [(64, 1024), (5, 320), (130, 512), (64, 8192)])
def test_mlp_workload(sol, batch, features):
    """The paper's MLP workload (three linear layers with ReLU, Sec. V) through the network object -- at reduced widths
    and at its real size (batch 64, 8192 features: the weight-streaming route that matrices of 16 MB and more take) --
    every layer element-wise against the checker on the checker's activations, and end to end."""
    wk = wl.config(5, batch=batch, hw=features)
    outs, _ = orc.network_forward(wk.layers, wk.params, wk.x, bf16=True, return_all=True)
    net, y = run_network(sol, wk)
    assert norm_err(y.reshape(outs[-1].shape), outs[-1]) <= TOL["bf16"]
    x = sol.to_device_nhwc(wk.x, sol.BF16)
    dev = [sol.to_device_nhwc(o if o.ndim == 4 else o[:, :, None, None], sol.BF16) for o in outs]
    nl = len(wk.layers)
    for i in range(nl - 1):
        net.layer_output(i).copy_(dev[i])
    for i in range(nl):
        net.run_layer(i, x)
        torch.cuda.synchronize()
        g = sol.to_host_nchw(net.y if i == nl - 1 else net.layer_output(i)).reshape(outs[i].shape)
        assert rel_err(g, outs[i]) <= TOL["bf16"], i
        if i < nl - 1:
            net.layer_output(i).copy_(dev[i])


# ---- stem convolution + max pool as one depth-first kernel ---------------------------------------------------------
STEM_POOL_CASES = [
    # N, H, W, pad      whole blocks, ragged pool blocks, odd conv extents (last pool window one row short), tiny images
    (2, 64, 64, 3), (1, 61, 75, 3), (3, 30, 44, 2), (2, 17, 19, 3), (1, 9, 9, 3), (1, 224, 224, 3),
]


@pytest.mark.parametrize("case", STEM_POOL_CASES, ids=lambda c: "x".join(map(str, c)))
def test_stem_pool_fused(sol, case):
    """7x7/2 stem + BN + ReLU + 3x3/2 pad-1 max pool in one kernel: against the checker, and bit for bit against
    the same library's two launches (convolution stored in bf16, then sol_pool)."""
    N, H, W, p = case
    rng = np.random.default_rng(1234 + H * W)
    pd = wl.pool_desc("max", 3, 2, 1)
    l, x, prm, _ = make_block(sol, rng, "bf16", N, 3, H, W, 64, 7, 2, p, pool=pd)
    want, _, _ = orc.fused_conv(x, prm, l, None, bf16=True)
    got, _, _ = run_block(sol, "bf16", l, x, prm, None)
    assert got.shape == want.shape
    assert rel_err(got, want) <= TOL["bf16"]
    conv_only, _, _ = run_block(sol, "bf16", dict(l, pool=None), x, prm, None)
    two, _ = sol.sol_pool(sol.to_device_nhwc(conv_only, sol.BF16), pd)
    torch.cuda.synchronize()
    assert np.array_equal(got, sol.to_host_nchw(two))


def test_stem_pool_fused_rejects_what_it_cannot_do(sol):
    rng = np.random.default_rng(5)
    pd = wl.pool_desc("max", 3, 2, 1)
    for kw in (dict(act="none"), dict(res=True), dict(K=32), dict(k=5)):
        K, k = kw.pop("K", 64), kw.pop("k", 7)
        l, x, prm, r = make_block(sol, rng, "bf16", 1, 3, 20, 20, K, k, 2, k // 2, pool=pd, **kw)
        with pytest.raises(sol.SolError) as e:
            run_block(sol, "bf16", l, x, prm, r)
        assert e.value.status == 6
    l, x, prm, r = make_block(sol, rng, "bf16", 1, 3, 20, 20, 64, 7, 2, 3, pool=pd)
    with pytest.raises(sol.SolError) as e:
        run_block(sol, "bf16", l, x, prm, r, want_argmax=True)
    assert e.value.status == 6
    with pytest.raises(sol.SolError) as e:                                   # average pool of that shape
        run_block(sol, "bf16", dict(l, pool=wl.pool_desc("avg", 3, 2, 1)), x, prm, r)
    assert e.value.status == 6


def test_network_fuses_stem_and_pool(sol):
    """A ResNet-shaped list without kept activations runs stem and pool as one launch (the pool layer reports the
    stem as its producer and launches nothing); same output as the plan that keeps every activation, bit for bit,
    and as the checker within tolerance."""
    wk = wl.config(2, batch=3, hw=64)
    outs, _ = orc.network_forward(wk.layers, wk.params, wk.x, bf16=True, return_all=True)
    net_keep, y_keep = run_network(sol, wk, keep=True)
    net, y = run_network(sol, wk, keep=False)
    kinds = [l["kind"] for l in wk.layers]
    assert kinds[0] == "conv" and kinds[1] == "pool"
    assert net.fused_into(1) == 0 and net.fused_into(0) == 0 and net.fused_into(2) == 2
    assert all(net_keep.fused_into(i) == i for i in range(len(kinds)))
    assert np.array_equal(y, y_keep)
    assert norm_err(y.reshape(outs[-1].shape), outs[-1]) <= TOL["bf16"]
    net.run_layer(1, sol.to_device_nhwc(wk.x, sol.BF16))                      # the elided layer: nothing to run, no error
    torch.cuda.synchronize()


# ---- projection shortcut inside the launch of the convolution that adds it -----------------------------------------------
@pytest.mark.parametrize("shape,cout", [((2, 64, 20, 24), 256), ((3, 64, 9, 7), 128), ((1, 64, 30, 30), 72)])
def test_projection_pair(sol, shape, cout):
    """x -> [1x1 64->64 + BN + ReLU -> 1x1 64->cout + BN] + [projection 1x1 64->cout + BN] -> ReLU: with kept activations
    three launches, without one launch for the last two; both against the checker, and against each other within one
    bf16 rounding of the shortcut."""
    c = wl.conv
    layers = [c(64, 3), c(64, 1, p=0, src=0), c(cout, 1, p=0, act="none", src=0), c(cout, 1, p=0, src=1, res=2), c(16, 1, p=0)]
    rng = np.random.default_rng(cout)
    x = _grid(rng.standard_normal((shape[0], 3, shape[2], shape[3])), "bf16")
    prm = wl.make_params(layers, 3, 31 + cout, bf16=True, bias_std=0.3)
    outs, _ = orc.network_forward(layers, prm, x, bf16=True, return_all=True)
    ys = {}
    for keep in (False, True):
        net = sol.Network(layers, x.shape, sol.BF16, flags=sol.NET_KEEP_ACTIVATIONS if keep else 0)
        net.set_params(prm)
        ys[keep] = sol.to_host_nchw(net.forward(sol.to_device_nhwc(x, sol.BF16)))
        torch.cuda.synchronize()
        assert [net.fused_into(i) for i in range(5)] == ([0, 1, 2, 3, 4] if keep else [0, 1, 3, 3, 4])
        if keep:
            got3 = sol.to_host_nchw(net.layer_output(3))
            assert rel_err(got3.reshape(outs[3].shape), outs[3]) <= TOL["bf16"]
    assert rel_err(ys[False].reshape(outs[-1].shape), outs[-1]) <= 2 * TOL["bf16"]
    # two bf16 results that differ by one rounding of the shortcut, seen through one more layer: ulp flips on both sides
    assert rel_err(ys[False], ys[True].astype(np.float64)) <= 2 * TOL["bf16"]
    assert norm_err(ys[False], ys[True].astype(np.float64)) <= TOL["bf16"] / 4


@pytest.mark.parametrize("cp,cm,stride,cout,hw", [(128, 64, 2, 256, (20, 24)), (64, 128, 1, 128, (9, 7)), (192, 64, 2, 72, (21, 19)),
                                                  (256, 128, 2, 512, (14, 14))])
def test_projection_pair_general(sol, cp, cm, stride, cout, hw):
    """The same pair with reductions of several 64-channel chunks and a strided shortcut (the shape of the first
    bottleneck of a later stage): x(cp) -> 1x1 cm -> 3x3/stride cm -> 1x1 cout (+ 1x1/stride shortcut of x) -> ReLU."""
    c = wl.conv
    layers = [c(cp, 3), c(cm, 1, p=0, src=0), c(cm, 3, s=stride, src=1), c(cout, 1, s=stride, p=0, act="none", src=0),
              c(cout, 1, p=0, src=2, res=3), c(16, 1, p=0)]
    rng = np.random.default_rng(cp + cout)
    x = _grid(rng.standard_normal((2, 3) + hw), "bf16")
    prm = wl.make_params(layers, 3, 77 + cout, bf16=True, bias_std=0.3)
    outs, _ = orc.network_forward(layers, prm, x, bf16=True, return_all=True)
    ys = {}
    for keep in (False, True):
        net = sol.Network(layers, x.shape, sol.BF16, flags=sol.NET_KEEP_ACTIVATIONS if keep else 0)
        net.set_params(prm)
        ys[keep] = sol.to_host_nchw(net.forward(sol.to_device_nhwc(x, sol.BF16)))
        torch.cuda.synchronize()
        assert [net.fused_into(i) for i in range(6)] == ([0, 1, 2, 3, 4, 5] if keep else [0, 1, 2, 4, 4, 5])
    assert rel_err(ys[False].reshape(outs[-1].shape), outs[-1]) <= 2 * TOL["bf16"]
    assert norm_err(ys[False], ys[True].astype(np.float64)) <= TOL["bf16"] / 4


# ---- channel concatenation, written in place by the producers where the plan allows ----------------------------------
def _concat_nets():
    c, cat, pool = wl.conv, wl.concat, wl.pool
    fire = lambda sq, ex: wl.fire_layers(1, 0, sq, ex)  # noqa: E731
    return {
        # name: (layers, (n, c, h, w), dtype, in-place parts per concat layer with flags 0)
        "fire_1x1_3x3": ([c(16, 3)] + fire(8, 16) + [c(8, 1, p=0)], (3, 3, 20, 24), "bf16", [2]),
        "fire_fp32": ([c(16, 3)] + fire(8, 16) + [c(8, 1, p=0)], (2, 3, 12, 12), "f32", [2]),
        "wide_1x1": ([c(256, 1, p=0)] + fire(64, 128) + [c(32, 1, p=0)], (4, 64, 28, 28), "bf16", [2]),
        "ragged_channels": ([c(16, 3)] + fire(8, 12) + [c(8, 1, p=0)], (2, 3, 10, 10), "bf16", [0]),      # 12 + 12: slices off the 16-byte grid
        "unequal_unaligned": ([c(16, 3), c(12, 1, p=0, src=0), c(20, 3, src=0), cat(1, 2), c(8, 1, p=0)], (2, 3, 10, 10), "bf16", [0]),
        "shared_producer": ([c(16, 3), c(16, 1, p=0, src=0), c(16, 3, src=0), cat(1, 2), c(8, 1, p=0, src=3), c(8, 1, p=0, src=1, res=4)],
                            (2, 3, 12, 12), "bf16", [1]),
        "pool_and_conv": ([c(16, 3), pool("max", 2, 2, 0), c(16, 3, s=2, src=0), cat(1, 2), c(8, 1, p=0)], (2, 3, 16, 16), "bf16", [1]),
        "concat_is_output": ([c(16, 3)] + fire(8, 16), (2, 3, 9, 11), "bf16", [2]),
        "nested": ([c(16, 3)] + fire(8, 16) + [c(32, 1, p=0, src=0), cat(4, 5), c(8, 1, p=0)], (2, 3, 12, 12), "bf16", [2, 2]),   # the second join extends the first: one shared buffer
    }


@pytest.mark.parametrize("name", sorted(_concat_nets()))
def test_concat_networks(sol, name):
    """Joins written in place by their producers, copied, or half and half: the plan's choice is as documented, the
    result is the same bits either way and matches the checker."""
    layers, shape, dt, want_parts = _concat_nets()[name]
    bf16 = dt == "bf16"
    rng = np.random.default_rng(len(name) * 7 + 3)
    x = _grid(rng.standard_normal(shape), dt)
    prm = wl.make_params(layers, shape[1], 4242, bf16=bf16, bias_std=0.3)
    outs, _ = orc.network_forward(layers, prm, x, bf16=bf16, return_all=True)
    d = _dt(sol, dt)
    res = {}
    for keep in (False, True):
        net = sol.Network(layers, shape, d, flags=sol.NET_KEEP_ACTIVATIONS if keep else 0)
        net.set_params(prm)
        y = sol.to_host_nchw(net.forward(sol.to_device_nhwc(x, d)))
        torch.cuda.synchronize()
        cats = [i for i, l in enumerate(layers) if l["kind"] == "concat"]
        parts = [net.concat_in_place(i) for i in cats]
        assert parts == (want_parts if not keep else [0] * len(cats)), (name, keep, parts)
        res[keep] = y
        if keep:
            for i in cats:
                got = sol.to_host_nchw(net.layer_output(i)) if i + 1 < len(layers) else y
                assert rel_err(got.reshape(outs[i].shape), outs[i]) <= TOL[dt]
    # in place or copied is the same arithmetic; the plan without kept activations may also pad channel counts to
    # multiples of 32 (other kernels, other accumulation order), hence a tolerance and not equality
    assert rel_err(res[False], res[True].astype(np.float64)) <= TOL[dt]
    assert rel_err(res[False].reshape(outs[-1].shape), outs[-1]) <= TOL[dt] * (4 if bf16 else 1)


def test_stem_writes_slices(sol):
    """The 7x7 stem kernel (interior and ragged blocks) and a 3x3 convolution as in-place producers of one join."""
    c = wl.conv
    for hw in (64, 50):
        # a 3-channel 1x1 layer in front, so that both stems can name one producer
        layers = [c(3, 1, p=0, bn=False, act="none"), c(64, 7, s=2, p=3, src=0), c(64, 3, s=2, p=1, src=0), wl.concat(1, 2), c(8, 1, p=0)]
        shape = (2, 3, hw, hw)
        x = _grid(np.random.default_rng(hw).standard_normal(shape), "bf16")
        prm = wl.make_params(layers, 3, 99, bf16=True, bias_std=0.3)
        outs, _ = orc.network_forward(layers, prm, x, bf16=True, return_all=True)
        ys = []
        for keep in (False, True):
            net = sol.Network(layers, shape, sol.BF16, flags=sol.NET_KEEP_ACTIVATIONS if keep else 0)
            net.set_params(prm)
            ys.append(sol.to_host_nchw(net.forward(sol.to_device_nhwc(x, sol.BF16))))
            assert net.concat_in_place(3) == (0 if keep else 2)
        assert np.array_equal(ys[0], ys[1])                 # no channel count here is padded: the same kernels, the same bits
        assert rel_err(ys[0].reshape(outs[-1].shape), outs[-1]) <= 4 * TOL["bf16"]


def test_squeezenet_shaped_network(sol):
    """Config 7 at a reduced size: every fire module's join is written in place; output against the checker."""
    wk = wl.config(7, batch=2, hw=96)
    outs, _ = orc.network_forward(wk.layers, wk.params, wk.x, bf16=True, return_all=True)
    net, y = run_network(sol, wk, keep=False)
    cats = [i for i, l in enumerate(wk.layers) if l["kind"] == "concat"]
    assert len(cats) == 8 and all(net.concat_in_place(i) == 2 for i in cats)
    _, y_keep = run_network(sol, wk, keep=True)
    assert norm_err(y, y_keep.astype(np.float64)) <= TOL["bf16"]     # squeeze outputs of 16 / 48 channels are padded to 32 / 64 in the lean plan
    assert norm_err(y.reshape(outs[-1].shape), outs[-1]) <= TOL["bf16"]
    assert norm_err(y_keep.reshape(outs[-1].shape), outs[-1]) <= TOL["bf16"]


# ---- depthwise convolution (the fusion engine's weighted pooling) -----------------------------------------------
def make_dw_block(rng, dt, N, C, H, W, k, sh, sw, p, bn=True, act="relu", res=False, bias_std=0.3):
    l = dict(wl.conv(C, k, 1, p, bn=bn, act=act, dw=True), sh=sh, sw=sw)
    x = _grid(rng.standard_normal((N, C, H, W)), dt)
    prm = {"w": _grid(rng.standard_normal((C, 1, k, k)) * np.sqrt(2.0 / (k * k)), dt),
           "bias": (rng.standard_normal(C) * bias_std).astype(np.float32)}
    if bn:
        prm.update(gamma=rng.uniform(0.5, 1.5, C).astype(np.float32), beta=rng.uniform(-0.1, 0.1, C).astype(np.float32),
                   mean=(rng.standard_normal(C) * 0.1).astype(np.float32), var=rng.uniform(0.5, 1.5, C).astype(np.float32))
    Ho, Wo = orc.out_size(H, k, sh, p), orc.out_size(W, k, sw, p)
    r = _grid(rng.standard_normal((N, C, Ho, Wo)), dt) if res else None
    return l, x, prm, r


def run_dw_block(sol, dt, l, x, prm, r):
    d = _dt(sol, dt)
    C = x.shape[1]
    cd = sol.ConvDesc(C, C, l["kh"], l["kw"], l["sh"], l["sw"], l["ph"], l["pw"])
    wp = sol.sol_pack_dwconv_weights(C, l["kh"], l["kw"], d, sol.dev_f32(prm["w"]))
    scale, shift = sol.sol_fold_bn(C, *(sol.dev_f32(prm[k]) if l["bn"] else None for k in ("gamma", "beta", "mean", "var")),
                                   sol.dev_f32(prm["bias"]), 1e-5)
    y = sol.sol_dwconv2d_fused(sol.to_device_nhwc(x, d), cd, wp, scale, shift,
                               sol.to_device_nhwc(r, d) if r is not None else None,
                               sol.ACT_RELU if l["act"] == "relu" else sol.ACT_NONE)
    torch.cuda.synchronize()
    return sol.to_host_nchw(y)


DW_CASES = [
    # N, C, H, W, k, sh, sw, p, res, bn, act     strip kernels (3x3, sw 1 / 2), ragged strips, tiles and channel groups
    (2, 32, 19, 17, 3, 1, 1, 1, False, True, "relu"),
    (3, 72, 14, 30, 3, 1, 1, 1, True, True, "relu"),
    (2, 64, 23, 23, 3, 2, 2, 1, False, True, "relu"),
    (1, 520, 9, 9, 3, 2, 2, 1, True, True, "none"),
    (2, 24, 11, 37, 3, 2, 1, 1, False, False, "relu"),     # vertical stride only
    (2, 16, 12, 9, 3, 1, 2, 0, False, True, "relu"),       # no padding, horizontal stride only
    (1, 1024, 7, 7, 3, 1, 1, 1, False, True, "relu"),
    (2, 8, 1, 1, 3, 1, 1, 1, False, True, "relu"),         # a single pixel: 8 of 9 taps are padding
    (1, 16, 3, 2, 3, 1, 1, 1, True, False, "none"),        # narrower than one strip
    (4, 128, 66, 70, 3, 1, 1, 1, False, True, "relu"),     # several row chunks per image, a short last chunk
    (2, 12, 31, 9, 3, 1, 1, 1, True, True, "relu"),        # three channel quads, ragged strip
    (3, 20, 29, 30, 3, 2, 2, 1, True, True, "relu"),
    (2, 64, 8, 8, 3, 2, 2, 0, False, True, "none"),        # stride 2 without padding: the last input row / column is unused
    # runtime-window kernel: other filters, channel counts that are no multiple of the vector width
    (2, 40, 13, 15, 5, 1, 1, 2, True, True, "relu"),
    (2, 16, 9, 10, 1, 1, 1, 0, False, True, "relu"),
    (3, 13, 10, 11, 3, 1, 1, 1, True, True, "relu"),
    (2, 6, 12, 12, 3, 2, 2, 1, False, False, "none"),
    (1, 8, 16, 16, 7, 3, 3, 3, False, True, "relu"),
]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("case", DW_CASES)
def test_dwconv_fused_matches_oracle(sol, dt, case):
    N, C, H, W, k, sh, sw, p, res, bn, act = case
    rng = np.random.default_rng(hash(case) % (2 ** 31))
    l, x, prm, r = make_dw_block(rng, dt, N, C, H, W, k, sh, sw, p, bn=bn, act=act, res=res)
    want, _, _ = orc.fused_conv(x, prm, l, r, bf16=(dt == "bf16"))
    got = run_dw_block(sol, dt, l, x, prm, r)
    assert rel_err(got, want) <= TOL[dt]


@pytest.mark.parametrize("stride", [1, 2])
def test_dwconv_long_row_walks(sol, stride):
    """Enough columns of work that every thread walks the maximum of 16 output rows (and a 1-row last chunk)."""
    rng = np.random.default_rng(5 + stride)
    H = 33 if stride == 1 else 65
    l, x, prm, r = make_dw_block(rng, "bf16", 64, 512, H, 64 * stride, 3, stride, stride, 1)
    want, _, _ = orc.fused_conv(x, prm, l, r, bf16=True)
    got = run_dw_block(sol, "bf16", l, x, prm, r)
    assert got.shape == (64, 512, 33, 64)
    assert rel_err(got, want) <= TOL["bf16"]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("geom", [(3, 1, 1), (3, 2, 1), (5, 1, 2)])
def test_dwconv_exact_integers(sol, dt, geom):
    """Small integers are exact in bf16 and their sums in fp32: the result must equal the checker's bit for bit,
    so a tap read from the wrong pixel or channel cannot hide inside a tolerance."""
    k, s, p = geom
    rng = np.random.default_rng(11)
    N, C, H, W = 2, 48, 21, 18
    l = wl.conv(C, k, s, p, bn=False, act="none", dw=True)
    x = rng.integers(-4, 5, (N, C, H, W)).astype(np.float32)
    prm = {"w": rng.integers(-3, 4, (C, 1, k, k)).astype(np.float32), "bias": rng.integers(-8, 9, C).astype(np.float32)}
    want, _, _ = orc.fused_conv(x, prm, l, None, bf16=(dt == "bf16"))
    got = run_dw_block(sol, dt, l, x, prm, None)
    assert np.array_equal(got, want)


def test_dwconv_empty_batch_and_errors(sol):
    d = sol.BF16
    wp = sol.sol_pack_dwconv_weights(16, 3, 3, d, torch.zeros((16, 1, 3, 3), device="cuda"))
    cd = sol.ConvDesc(16, 16, 3, 3, 1, 1, 1, 1)
    y = sol.sol_dwconv2d_fused(torch.empty((0, 8, 8, 16), dtype=torch.bfloat16, device="cuda"), cd, wp)
    assert y.shape == (0, 8, 8, 16)
    x = torch.zeros((1, 8, 8, 16), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sol.SolError):          # a depthwise convolution keeps the channel count
        sol.sol_dwconv2d_fused(x, sol.ConvDesc(32, 16, 3, 3, 1, 1, 1, 1), wp)
    with pytest.raises(sol.SolError):          # filter larger than the padded input
        sol.sol_dwconv2d_fused(x, sol.ConvDesc(16, 16, 11, 11, 1, 1, 0, 0), wp)
    with pytest.raises(sol.SolError):          # missing weights
        sol.sol_dwconv2d_fused(x, cd, None)
    with pytest.raises(sol.SolError):          # depthwise layers are inference-only
        sol.Network([wl.conv(16, 3, dw=True), wl.gap(), wl.linear(4)], (2, 16, 8, 8), d, flags=sol.NET_TRAINING)
    with pytest.raises(sol.SolError):          # channel count must be kept
        sol.Network([wl.conv(24, 3, dw=True)], (2, 16, 8, 8), d)


def test_full_size_depthwise_layers(sol):
    """Every distinct depthwise geometry of the separable chain at the full benchmark batch, in the launch
    configuration the planner uses, against the checker's full output (the checker's plain loops finish a
    layer in seconds: there is no reduction over channels)."""
    wk = wl.config(6)
    ch, hw, seen = wk.in_shape[1], wk.in_shape[2], set()
    rng = np.random.default_rng(wk.seed)
    for i, l in enumerate(wk.layers):
        if l["kind"] != "conv":
            break
        key = (ch, hw, l["sh"])
        if l.get("dw") and key not in seen:
            seen.add(key)
            x = wl.to_bf16_grid(rng.standard_normal((wk.in_shape[0], ch, hw, hw), dtype=np.float32))
            want, _, _ = orc.fused_conv(x, wk.params[i], l, None, bf16=True)
            got = run_dw_block(sol, "bf16", l, x, wk.params[i], None)
            err = rel_err(got, want)
            print(f"  L{i} C{ch} {hw}x{hw} s{l['sh']}: rel err {err:.3e}", flush=True)
            assert err <= TOL["bf16"], (i, key, err)
            del x, want, got
        ch, hw = l["cout"], orc.out_size(hw, l["kh"], l["sh"], l["ph"])
    assert len(seen) == 9
