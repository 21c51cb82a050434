"""Parity of the depth-first expand -> reduce pair (sol_expand_reduce_fused, and the network plans that use it: the
last 1x1 convolution of one bottleneck and the first 1x1 convolution of the next in one launch) against the CPU
checker, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle as orc
from paper_2003_10688_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
WM = 256


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


def _norm_err(g, r):
    return float(np.linalg.norm(np.asarray(g, np.float64) - r) / max(np.linalg.norm(r), 1e-30))


def _case(rng, N, H, W, C4, bias_std=0.3, WZ=256):
    t = wl.to_bf16_grid(rng.standard_normal((N, WM, H, W)))
    r = wl.to_bf16_grid(rng.standard_normal((N, C4, H, W)))
    ls = [wl.conv(C4, 1, p=0), wl.conv(WZ, 1, p=0)]
    prm = []
    for l, cin in zip(ls, (WM, C4)):
        prm.append({"w": wl.to_bf16_grid(rng.standard_normal((l["cout"], cin, 1, 1)) * np.sqrt(2.0 / cin)),
                    "bias": (rng.standard_normal(l["cout"]) * bias_std).astype(np.float32),
                    "gamma": rng.uniform(0.5, 1.5, l["cout"]).astype(np.float32), "beta": rng.uniform(-0.1, 0.1, l["cout"]).astype(np.float32),
                    "mean": (rng.standard_normal(l["cout"]) * 0.1).astype(np.float32), "var": rng.uniform(0.5, 1.5, l["cout"]).astype(np.float32)})
    return t, r, ls, prm


def _gpu(sol, t, r, ls, prm, fold=True):
    args = []
    for l, p, cin in zip(ls, prm, (WM, ls[0]["cout"])):
        cd = sol.ConvDesc(l["cout"], cin, 1, 1, 1, 1, 0, 0)
        wp = sol.sol_pack_conv_weights(cd, sol.BF16, sol.dev_f32(p["w"]))
        if fold:
            sc, sh = sol.sol_fold_bn(l["cout"], *(sol.dev_f32(p[k]) for k in ("gamma", "beta", "mean", "var")), sol.dev_f32(p["bias"]), 1e-5)
        else:
            sc, sh = torch.ones(l["cout"], device="cuda:0"), sol.dev_f32(p["bias"])
        args.append((wp, sc, sh))
    (w3, s3, h3), (w1, s1, h1) = args
    y, z = sol.sol_expand_reduce_fused(sol.to_device_nhwc(t, sol.BF16), ls[0]["cout"], w3, s3, h3, sol.to_device_nhwc(r, sol.BF16), ls[1]["cout"], w1, s1, h1)
    torch.cuda.synchronize()
    return sol.to_host_nchw(y), sol.to_host_nchw(z)


def _ref(t, r, ls, prm):
    y, _, _ = orc.fused_conv(t, prm[0], ls[0], residual=r, bf16=True)
    z, _, _ = orc.fused_conv(y, prm[1], ls[1], bf16=True)
    return y, z


XR_CASES = [
    # N, H, W, C4      one tile; several tiles over several XCDs with idle workgroups at the end of the grid; every pass count
    (1, 8, 8, 1024), (5, 16, 16, 1024), (2, 8, 16, 512), (3, 8, 8, 128), (7, 4, 16, 640), (16, 14, 14, 1024),
    # ragged last tile: 196 = 3 * 64 + 4 pixels, 49 pixels (less than a tile), 5 * 81 = 405 = 6 * 64 + 21
    (1, 14, 14, 1024), (1, 7, 7, 512), (5, 9, 9, 256),
    # 512 output channels (the pair across a stage border): the second contraction runs one 32-channel group per stage
    (1, 8, 8, 1024, 512), (5, 16, 16, 1024, 512), (3, 8, 8, 128, 512), (7, 4, 16, 640, 512), (1, 14, 14, 1024, 512), (5, 9, 9, 256, 512),
]


@pytest.mark.parametrize("case", XR_CASES, ids=lambda c: "x".join(map(str, c)))
def test_expand_reduce_fused_matches_oracle(sol, case):
    """Both outputs of the pair kernel against the checker's two fused layers (the first rounding its stored output to
    bf16, as the kernel rounds y where it parks it for the second contraction), element-wise."""
    N, H, W, C4 = case[:4]
    WZ = case[4] if len(case) > 4 else 256
    rng = np.random.default_rng(300 + H * W + C4 + WZ - 256)
    t, r, ls, prm = _case(rng, N, H, W, C4, WZ=WZ)
    print(f"expand-reduce {case}", flush=True)
    gy, gz = _gpu(sol, t, r, ls, prm)
    wy, wz = _ref(t, r, ls, prm)
    ey, ez = rel_err(gy, wy), rel_err(gz, wz)
    print(f"expand-reduce {case}: rel err y {ey:.3e}, z {ez:.3e}")
    assert ey <= TOL["bf16"] and ez <= TOL["bf16"], (case, ey, ez)


def test_expand_reduce_fused_exact_integers(sol):
    """Small-integer inputs and sparse +-1 weights, unit scales: every intermediate is exact in bf16 and in fp32, so the
    kernel must reproduce the checker bit for bit (channel order of both contractions, pass order, shortcut, stores)."""
    rng = np.random.default_rng(6)
    for (N, H, W, C4, WZ) in [(2, 8, 8, 1024, 256), (1, 8, 24, 384, 256), (2, 8, 8, 1024, 512), (1, 9, 9, 256, 512)]:
        t = rng.integers(-2, 3, (N, WM, H, W)).astype(np.float32)
        r = rng.integers(-3, 4, (N, C4, H, W)).astype(np.float32)
        ls = [wl.conv(C4, 1, p=0, bn=False), wl.conv(WZ, 1, p=0, bn=False)]
        prm = []
        for l, cin in zip(ls, (WM, C4)):
            w = np.zeros((l["cout"], cin, 1, 1), np.float32)
            idx = rng.random(w.shape) < (4.0 / cin)                     # about four non-zero taps per output channel
            w[idx] = rng.choice([-1.0, 1.0], int(idx.sum()))
            prm.append({"w": w, "bias": rng.integers(-1, 2, l["cout"]).astype(np.float32)})
        print(f"expand-reduce exact {N, H, W, C4}", flush=True)
        gy, gz = _gpu(sol, t, r, ls, prm, fold=False)
        wy, wz = _ref(t, r, ls, prm)
        assert np.abs(wy).max() < 256 and np.array_equal(wy, np.round(wy)) and np.abs(wz).max() < 256     # integers that bf16 holds exactly
        assert np.array_equal(gy, wy), (N, H, W, C4, np.count_nonzero(gy != wy))
        assert np.array_equal(gz, wz), (N, H, W, C4, np.count_nonzero(gz != wz))


def test_expand_reduce_fused_rejects_what_it_cannot_do(sol):
    z = torch.zeros(1024, device="cuda:0")
    bf = dict(dtype=torch.bfloat16, device="cuda:0")

    def call(t, c4, r, cz=256):
        return sol.sol_expand_reduce_fused(t, c4, z, z, z, r, cz, z, z, z)

    for t, c4, r, cz in [(torch.zeros((1, 8, 8, 128), **bf), 512, torch.zeros((1, 8, 8, 512), **bf), 256),      # 128 input channels
                         (torch.zeros((1, 8, 8, 256), **bf), 2048, torch.zeros((1, 8, 8, 2048), **bf), 256),    # too wide
                         (torch.zeros((1, 8, 8, 256), **bf), 1024, torch.zeros((1, 8, 8, 1024), **bf), 384),    # 384 output channels
                         (torch.zeros((1, 8, 8, 256), device="cuda:0"), 1024, torch.zeros((1, 8, 8, 1024), device="cuda:0"), 256)]:   # fp32
        with pytest.raises(sol.SolError) as e:
            call(t, c4, r, cz)
        assert e.value.status in (3, 6), e.value.status
    y, zz = call(torch.zeros((0, 8, 8, 256), **bf), 1024, torch.zeros((0, 8, 8, 1024), **bf))
    assert tuple(y.shape) == (0, 8, 8, 1024) and tuple(zz.shape) == (0, 8, 8, 256)


# ---- the plan runs expand -> reduce pairs as one launch -----------------------------------------------------------------
def test_network_runs_expand_reduce_pairs(sol):
    """ResNet-50-shaped list at 128x128 input (the 14x14 stage becomes 8x8), lean plan: (a) each
    pair, fed the checker's inputs, gives the checker's two outputs element-wise (2e-2); (b) the whole pass agrees with the
    layer-by-layer plan and with the checker norm-wise; (c) the plan reports what it fused; (d) a recorded graph of the
    fused plan replays bit-identically."""
    wk = wl.config(3, batch=3, hw=128)
    L = wk.layers
    outs, _ = orc.network_forward(L, wk.params, wk.x, bf16=True, return_all=True)
    x = sol.to_device_nhwc(wk.x, sol.BF16)
    net = sol.Network(L, wk.in_shape, sol.BF16)
    net.set_params(wk.params)
    starts = [i for i in range(len(L)) if net.xr_state(i) >= 0]
    assert len(starts) == 5, starts                # bottlenecks 2-6 of the 1024-channel stage, each with the reduce layer behind it (the last one's has 512 channels)
    assert all(net.xr_state(i) == 0 for i in starts)     # three tiles of 64 pixels: the plan's heuristic leaves such pairs alone
    for i in starts:
        net.set_xr(i, 0)
        assert net.fused_into(i + 1) == i + 1
    y_plain = sol.to_host_nchw(net.forward(x)).copy()
    for i in starts:
        net.set_xr(i, 1)
        assert net.xr_state(i) == 1 and net.fused_into(i + 1) == i and net.fused_into(i) == i
    y_fused = sol.to_host_nchw(net.forward(x)).copy()
    torch.cuda.synchronize()
    assert _norm_err(y_fused, y_plain.astype(np.float64)) <= TOL["bf16"]
    assert _norm_err(y_fused.reshape(outs[-1].shape), outs[-1]) <= TOL["bf16"]
    worst = 0.0
    for i in starts:                               # teacher-forced: the checker's tensors in the producers' buffers
        for j in (L[i]["res"], i - 1):
            net.layer_output(j).copy_(sol.to_device_nhwc(outs[j], sol.BF16))
        net.run_layer(i, x)
        net.run_layer(i + 1, x)                    # launches nothing
        torch.cuda.synchronize()
        for j in (i, i + 1):
            e = rel_err(sol.to_host_nchw(net.layer_output(j)), outs[j])
            worst = max(worst, e)
            assert e <= TOL["bf16"], (i, j, e)
    print(f"fused expand-reduce pairs {starts}: worst element-wise rel err {worst:.3e}")
    side = torch.cuda.Stream()
    launch = net.graph(x, side)
    eager = net.forward(x).clone()
    torch.cuda.synchronize()
    for _ in range(3):
        net.y.zero_()
        torch.cuda.synchronize()
        yg = launch()
        side.synchronize()
        assert torch.equal(yg, eager)
    with pytest.raises(sol.SolError) as e:         # starts no pair
        net.set_xr(0, 1)
    assert e.value.status == 6


def test_autotune_chooses_between_pair_and_layers(sol):
    wk = wl.config(3, batch=4, hw=128)
    outs, _ = orc.network_forward(wk.layers, wk.params, wk.x, bf16=True, return_all=True)
    net = sol.Network(wk.layers, wk.in_shape, sol.BF16)
    net.set_params(wk.params)
    x = sol.to_device_nhwc(wk.x, sol.BF16)
    tuned = net.autotune(x, reps=2)
    pairs = {k: v for k, v in tuned.items() if str(k).endswith("x")}
    assert len(pairs) == 5 and all(v in (0, 1) for v in pairs.values()), tuned
    y = sol.to_host_nchw(net.forward(x))
    assert _norm_err(y.reshape(outs[-1].shape), outs[-1]) <= TOL["bf16"]
    net2 = sol.Network(wk.layers, wk.in_shape, sol.BF16)      # the saved plan restores the same launches
    net2.set_params(wk.params)
    net2.set_tiles(tuned)
    assert np.array_equal(sol.to_host_nchw(net2.forward(x)), y)


def test_full_size_expand_reduce_pairs_sampled(sol):
    """The pair launches of the benchmark's pass (batch 64, 14x14, 256 -> 1024 -> 256 or 512 channels), in the network object
    with its lean plan: random stored inputs, both outputs checked at sampled pixels -- y at sampled (pixel, channel)
    points; z from the checker's y at ALL channels of the sampled pixels."""
    wk = wl.config(3)
    L, P = wk.layers, wk.params
    net = sol.Network(L, wk.in_shape, sol.BF16)
    net.set_params(P)
    x = sol.to_device_nhwc(wk.x[:1].repeat(wk.in_shape[0], 0), sol.BF16)
    starts = [i for i in range(len(L)) if net.xr_state(i) == 1]
    assert len(starts) == 5 and [L[i + 1]["cout"] for i in starts] == [256] * 4 + [512]
    rng = np.random.default_rng(77)
    N, H, W = wk.in_shape[0], 14, 14
    for i in starts:
        print(f"full-size expand-reduce pair L{i}+L{i + 1}", flush=True)
        t = wl.to_bf16_grid(rng.standard_normal((N, WM, H, W), dtype=np.float32))
        r = wl.to_bf16_grid(rng.standard_normal((N, 1024, H, W), dtype=np.float32))
        net.layer_output(i - 1).copy_(sol.to_device_nhwc(t, sol.BF16))
        net.layer_output(L[i]["res"]).copy_(sol.to_device_nhwc(r, sol.BF16))
        net.run_layer(i, x)
        torch.cuda.synchronize()
        gy, gz = sol.to_host_nchw(net.layer_output(i)), sol.to_host_nchw(net.layer_output(i + 1))
        assert gy.shape == (N, 1024, H, W) and gz.shape == (N, L[i + 1]["cout"], H, W)
        pix = np.stack([rng.integers(0, s, 48) for s in (N, H, W)], 1)
        pix[:3] = [[0, 0, 0], [N - 1, H - 1, W - 1], [N // 2, 0, W - 1]]
        coords = np.array([[n, k, h, w] for (n, h, w) in pix for k in range(1024)], np.int32)
        wy = orc.fused_conv_points(t, P[i], L[i], coords, r, bf16=True).reshape(len(pix), 1024)
        g = gy[coords[:, 0], coords[:, 1], coords[:, 2], coords[:, 3]].reshape(len(pix), 1024)
        ey = rel_err(g, wy)
        ysmall = np.ascontiguousarray(wy.T[None, :, None, :])                  # [1, 1024, 1, pixels]: the 1x1 convolution sees pixels only
        wz, _, _ = orc.fused_conv(ysmall, P[i + 1], L[i + 1], bf16=True)
        gzs = np.stack([gz[n, :, h, w] for (n, h, w) in pix], 1)[None, :, None, :]
        ez = rel_err(gzs, wz)
        print(f"  pair L{i}+L{i + 1}: y {ey:.3e}, z {ez:.3e}")
        assert ey <= TOL["bf16"] and ez <= TOL["bf16"], (i, ey, ez)
