"""The forward pass that allocates nothing (sol_network_forward_static: activations in a static device array of the
library) against sol_network_forward with a caller workspace, through the C ABI: two calls in a row, the second on a
smaller network, so that the second finds the first one's leftovers in the shared array."""
import numpy as np
import pytest
import torch

import oracle as orc
from paper_2003_10688_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_static_workspace_forward_matches_the_workspace_forward():
    from paper_2003_10688_amd import sol

    sol.lib()
    results = []
    for cfg, batch, hw, dt in ((1, 16, 32, sol.F32), (3, 2, 64, sol.BF16), (1, 3, 20, sol.F32)):   # large, other dtype + pairs, smaller
        wk = wl.config(cfg, batch=batch, hw=hw)
        net = sol.Network(wk.layers, wk.in_shape, dt)
        net.set_params(wk.params)
        x = sol.to_device_nhwc(wk.x, dt)
        want = net.forward(x).clone()
        torch.cuda.synchronize()
        net.y.zero_()
        net.workspace.fill_(0x7f)              # the static pass must not depend on the caller's workspace
        got = net.forward_static(x).clone()
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"cfg{cfg} batch {batch}: static-workspace pass differs from the workspace pass"
        results.append((wk, sol.to_host_nchw(got)))
    # and against the checker (fp32 configs: 1e-4 element-wise)
    for wk, got in results:
        if wk.bf16:
            continue
        ref = orc.network_forward(wk.layers, wk.params, wk.x)
        err = float(np.max(np.abs(got.reshape(ref.shape) - ref) / np.maximum(np.abs(ref), np.sqrt(np.mean(ref * ref)))))
        assert err <= 1e-4, err


def test_static_workspace_forward_rejects_what_does_not_fit():
    from paper_2003_10688_amd import sol

    wk = wl.config(3, batch=8, hw=224)         # about 77 MB of activations: beyond the static array
    net = sol.Network(wk.layers, wk.in_shape, sol.BF16)
    assert sol.lib().sol_network_workspace_bytes(net._h) > 32 << 20
    x = torch.zeros((8, 224, 224, 3), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(sol.SolError) as e:
        net.forward_static(x)
    assert e.value.status == 5
    tnet = sol.Network([wl.conv(8, 3), wl.gap(), wl.linear(4)], (2, 3, 8, 8), sol.F32, flags=sol.NET_TRAINING)
    with pytest.raises(sol.SolError) as e:
        tnet.forward_static(torch.zeros((2, 8, 8, 3), device="cuda:0"))
    assert e.value.status == 6
