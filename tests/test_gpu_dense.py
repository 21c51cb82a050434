"""Parity of the pre-activation convolution (BN + ReLU on the input side, sol_conv2d_preact_fused) and of the
DenseNet-shaped plans (dense chains sharing one buffer) against the CPU checker, through the C ABI."""
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


def norm_err(g, r):
    return float(np.linalg.norm(np.asarray(g, np.float64) - r) / max(np.linalg.norm(r), 1e-30))


def _grid(a, dt):
    return wl.to_bf16_grid(a) if dt == "bf16" else np.asarray(a, np.float32)


PRE_CASES = [
    # N, Ctot, C (prefix read), H, W, K, k, s, p, pool, res
    (2, 64, 64, 13, 11, 128, 1, 1, 0, None, False),       # dense input, 1x1
    (2, 256, 96, 9, 10, 128, 1, 1, 0, None, False),       # channel prefix, not a whole reduction chunk: masked channels
    (1, 192, 160, 14, 14, 40, 1, 1, 0, "avg", False),     # transition-like: fused 2x2 average pool, ragged Cout
    (2, 64, 64, 10, 9, 32, 3, 1, 1, None, True),          # 3x3 with padding: border taps are 0, not relu(shift); residual
    (3, 32, 24, 7, 7, 16, 3, 2, 1, None, False),          # prefix of 24 channels: element-gather path
    (1, 128, 128, 6, 6, 256, 1, 2, 0, "max", False),      # strided 1x1 + fused max pool
]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("case", PRE_CASES, ids=lambda c: "x".join(map(str, c)))
def test_preact_conv_matches_oracle(sol, dt, case):
    N, Ctot, Cc, H, W, K, k, s, p, pool, with_res = case
    rng = np.random.default_rng(7 + Ctot + K)
    d = sol.BF16 if dt == "bf16" else sol.F32
    xfull = _grid(rng.standard_normal((N, Ctot, H, W)), dt)
    if Cc < Ctot:
        xfull[:, Cc:] = np.nan                                  # what lies behind the prefix must never be looked at
    l = wl.conv(K, k, s, p, pre_bn=True, pool=wl.pool_desc(pool, 2, 2, 0) if pool else None)
    prm = {"w": _grid(rng.standard_normal((K, Cc, k, k)) * np.sqrt(2.0 / (Cc * k * k)), dt), "bias": (rng.standard_normal(K) * 0.3).astype(np.float32),
           "gamma": rng.uniform(0.5, 1.5, K).astype(np.float32), "beta": rng.uniform(-0.1, 0.1, K).astype(np.float32),
           "mean": (rng.standard_normal(K) * 0.1).astype(np.float32), "var": rng.uniform(0.5, 1.5, K).astype(np.float32),
           "pre_gamma": rng.uniform(0.5, 1.5, Cc).astype(np.float32), "pre_beta": rng.uniform(0.2, 0.6, Cc).astype(np.float32),
           "pre_mean": (rng.standard_normal(Cc) * 0.1).astype(np.float32), "pre_var": rng.uniform(0.5, 1.5, Cc).astype(np.float32)}
    Ho, Wo = orc.out_size(H, k, s, p), orc.out_size(W, k, s, p)
    r = _grid(rng.standard_normal((N, K, Ho, Wo)), dt) if with_res else None
    want, _, _ = orc.fused_conv(xfull[:, :Cc], prm, l, r, bf16=dt == "bf16")
    cd = sol.ConvDesc(K, Cc, k, k, s, s, p, p)
    wp = sol.sol_pack_conv_weights(cd, d, sol.dev_f32(prm["w"]))
    sc, sh = sol.sol_fold_bn(K, *(sol.dev_f32(prm[q]) for q in ("gamma", "beta", "mean", "var")), sol.dev_f32(prm["bias"]), 1e-5)
    psc, psh = sol.sol_fold_bn(Cc, *(sol.dev_f32(prm[q]) for q in ("pre_gamma", "pre_beta", "pre_mean", "pre_var")), None, 1e-5)
    y = sol.sol_conv2d_preact_fused(sol.to_device_nhwc(xfull, d), cd, wp, psc, psh, sc, sh, sol.to_device_nhwc(r, d) if r is not None else None,
                                    sol.ACT_RELU, l["pool"], channels=Cc)
    torch.cuda.synchronize()
    got = sol.to_host_nchw(y)
    assert not np.isnan(got).any()
    err = rel_err(got, want)
    print(f"preact {case} {dt}: rel err {err:.3e}")
    assert err <= TOL[dt], (case, dt, err)


def _small_densenet():
    return wl.densenet_layers(num_classes=10, growth=16, blocks=(2, 4, 2), stem=32, bottleneck=2)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_densenet_shaped_network(sol, dt):
    """A small DenseNet-shaped list (three dense blocks of 2, 4 and 2 layers, two transitions; every width a multiple of 8): the lean plan keeps every dense block in one
    buffer (all joins in place but the block input), every layer matches the checker on the checker's activations
    (kept plan, element-wise), the lean and the kept plan agree, and the whole pass matches end to end."""
    layers = _small_densenet()
    bf = dt == "bf16"
    N, hw = 3, 48
    params = wl.make_params(layers, 3, 77, bf, bias_std=0.2)
    x = wl.make_input((N, 3, hw, hw), 78, "normal", bf)
    d = sol.BF16 if bf else sol.F32
    outs, _ = orc.network_forward(layers, params, x, bf16=bf, return_all=True)
    xd = sol.to_device_nhwc(x, d)
    keep = sol.Network(layers, x.shape, d, flags=sol.NET_KEEP_ACTIVATIONS)
    keep.set_params(params)
    y_keep = sol.to_host_nchw(keep.forward(xd)).copy()
    nl = len(layers)
    dev = [sol.to_device_nhwc(o if o.ndim == 4 else o[:, :, None, None], d) for o in outs]
    for i in range(nl - 1):
        keep.layer_output(i).copy_(dev[i])
    errs = []
    for i in range(nl):
        keep.run_layer(i, xd)
        torch.cuda.synchronize()
        g = sol.to_host_nchw(keep.y if i == nl - 1 else keep.layer_output(i)).reshape(outs[i].shape)
        errs.append(rel_err(g, outs[i]))
        if i < nl - 1:
            keep.layer_output(i).copy_(dev[i])
    print(f"densenet-shaped {dt}: layer-by-layer max rel err {max(errs):.3e}")
    assert max(errs) <= TOL[dt], errs
    lean = sol.Network(layers, x.shape, d)
    lean.set_params(params)
    y_lean = sol.to_host_nchw(lean.forward(xd)).copy()
    torch.cuda.synchronize()
    cats = [i for i, l in enumerate(layers) if l["kind"] == "concat"]
    parts = [lean.concat_in_place(i) for i in cats]
    heads = [i for i in cats if layers[layers[i]["src"]]["kind"] != "concat"]
    assert all(p == (1 if i in heads else 2) for i, p in zip(cats, parts)), (cats, parts, heads)
    assert [keep.concat_in_place(i) for i in cats] == [0] * len(cats)
    if bf:
        assert norm_err(y_lean, y_keep.astype(np.float64)) <= TOL[dt]
        assert norm_err(y_lean.reshape(outs[-1].shape), outs[-1]) <= TOL[dt]
    else:
        assert rel_err(y_lean, y_keep) <= TOL[dt]
        assert rel_err(y_lean.reshape(outs[-1].shape), outs[-1]) <= TOL[dt]
    y2 = sol.to_host_nchw(lean.forward(xd))
    assert np.array_equal(y2, y_lean)                       # run-to-run identical
    tuned = lean.autotune(xd, reps=2)
    y3 = sol.to_host_nchw(lean.forward(xd))
    assert (norm_err if bf else rel_err)(y3.reshape(outs[-1].shape), outs[-1]) <= TOL[dt], tuned


def test_preact_api_errors(sol):
    x = torch.zeros((1, 5, 5, 64), dtype=torch.bfloat16, device="cuda:0")
    cd = sol.ConvDesc(32, 48, 1, 1, 1, 1, 0, 0)
    wp = sol.sol_pack_conv_weights(cd, sol.BF16, sol.dev_f32(np.zeros((32, 48, 1, 1), np.float32)))
    z = torch.zeros(64, device="cuda:0")
    with pytest.raises(sol.SolError) as e:                     # scale without shift
        sol.sol_conv2d_preact_fused(x, cd, wp, z, None, channels=48)
    assert e.value.status == 1
    y = sol.sol_conv2d_preact_fused(x, cd, wp, z, z, channels=48)
    assert tuple(y.shape) == (1, 5, 5, 32)
    with pytest.raises(sol.SolError) as e:                     # a training network with an input-side BN
        sol.Network([wl.conv(8, 3), wl.conv(8, 1, p=0, pre_bn=True), wl.gap(), wl.linear(4)], (2, 3, 8, 8), sol.F32, flags=sol.NET_TRAINING)
    assert e.value.status == 6
