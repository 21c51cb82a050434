"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares, and its
host-side logic (argument validation, shape inference, buffer planning) behaves -- no kernel runs."""
import ctypes as C
import os
import re

import pytest

from paper_2003_10688_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sol():
    from paper_2003_10688_amd import sol as s

    if not os.path.exists(s.LIB_PATH):
        from paper_2003_10688_amd import build

        build.build(verbose=False)
    s.lib()
    return s


def test_exports_every_declared_symbol(sol):
    hdr = open(os.path.join(ROOT, "include", "sol.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(sol_[a-z0-9_]+)\s*\(", hdr))
    assert {"sol_conv2d_fused", "sol_linear", "sol_pool", "sol_network_forward", "sol_network_create"} <= names
    for n in sorted(names):
        assert hasattr(sol.lib(), n), f"{n} declared in include/sol.h but not exported"
    assert b"gfx950" in sol.lib().sol_version()


def test_out_size_and_packed_bytes(sol):
    assert sol.sol_out_size(224, 7, 2, 3) == 112 and sol.sol_out_size(112, 3, 2, 1) == 56
    assert sol.sol_out_size(5, 2, 2, 0) == 2 and sol.sol_out_size(7, 3, 1, 1) == 7
    assert sol.sol_packed_weight_bytes(sol.ConvDesc(64, 3, 7, 7, 2, 2, 3, 3), sol.BF16) == 64 * 192 * 2   # 147 -> 192
    assert sol.sol_packed_weight_bytes(sol.ConvDesc(64, 3, 7, 7, 2, 2, 3, 3), sol.F32) == 64 * 160 * 4    # 147 -> 160
    assert sol.sol_packed_weight_bytes(sol.ConvDesc(256, 64, 1, 1, 1, 1, 0, 0), sol.BF16) == 256 * 64 * 2


def _status(sol, fn, *args):
    return fn(*args)


def test_validation_rejects_before_launch(sol):
    L = sol.lib()
    xd = sol.TensorDesc(1, 8, 8, 16, sol.F32)
    cd = sol.ConvDesc(8, 16, 3, 3, 1, 1, 1, 1)
    null = C.c_void_p(0)
    fake = C.c_void_p(0x1000)          # never dereferenced: validation fails first
    call = lambda xd_, x, cd_, w, y, pool=None: L.sol_conv2d_fused(  # noqa: E731
        C.byref(xd_), x, C.byref(cd_), w, null, null, null, 0, C.byref(pool) if pool else None, y, null, null, null)
    assert call(xd, null, cd, fake, fake) == 1                                            # NULL x
    assert b"NULL" in L.sol_last_error()
    assert call(xd, fake, sol.ConvDesc(8, 4, 3, 3, 1, 1, 1, 1), fake, fake) == 2           # cin mismatch
    assert call(xd, fake, sol.ConvDesc(8, 16, 3, 3, 0, 1, 1, 1), fake, fake) == 2          # zero stride
    assert call(sol.TensorDesc(1, 8, 8, 16, 7), fake, cd, fake, fake) == 3                 # dtype
    assert call(xd, C.c_void_p(0x1004), cd, fake, fake) == 4                               # alignment
    assert call(xd, fake, cd, fake, fake, sol.PoolDesc(sol.POOL_MAX, 3, 3, 2, 2, 1, 1, 1)) == 6   # unfusable pool
    assert call(sol.TensorDesc(1, 2, 2, 16, 0), fake, sol.ConvDesc(8, 16, 5, 5, 1, 1, 0, 0), fake, fake) == 2  # filter > input
    big = sol.TensorDesc(65536, 512, 512, 16, sol.BF16)                                    # >= 2^31 elements
    assert call(big, fake, cd, fake, fake) == 6
    assert L.sol_pool(C.byref(xd), fake, C.byref(sol.PoolDesc(sol.POOL_MAX, 2, 2, 2, 2, 2, 2, 1)), fake, null, null) == 2
    assert L.sol_linear(4, 0, 3, 0, fake, fake, null, 0, fake, null) == 2


def _create(sol, layers, shape, dt, flags=0):
    h = C.c_void_p(0)
    n, c, hh, ww = shape
    st = sol.lib().sol_network_create(sol.make_layer_array(layers), len(layers), C.byref(sol.TensorDesc(n, hh, ww, c, dt)),
                                      flags, C.byref(h))
    return st, h


def test_planner_shapes_and_buffers(sol):
    L = sol.lib()
    wk = wl.config(3)
    st, h = _create(sol, wk.layers, wk.in_shape, sol.BF16)
    assert st == 0
    d = sol.TensorDesc()
    assert L.sol_network_output_desc(h, -1, C.byref(d)) == 0 and (d.n, d.h, d.w, d.c) == (64, 1, 1, 1000)
    assert L.sol_network_output_desc(h, 0, C.byref(d)) == 0 and (d.n, d.h, d.w, d.c) == (64, 112, 112, 64)
    assert L.sol_network_output_desc(h, 1, C.byref(d)) == 0 and (d.n, d.h, d.w, d.c) == (64, 56, 56, 64)
    assert L.sol_network_output_desc(h, len(wk.layers) - 3, C.byref(d)) == 0 and (d.n, d.h, d.w, d.c) == (64, 7, 7, 2048)
    assert L.sol_network_num_layers(h) == len(wk.layers)
    ws = L.sol_network_workspace_bytes(h)
    biggest = 64 * 56 * 56 * 256 * 2                      # largest live activation
    assert 2 * biggest <= ws <= 5 * biggest               # buffers are reused, not one per layer
    pb = L.sol_network_param_bytes(h)
    assert 25.5e6 * 2 <= pb <= 25.5e6 * 2 * 1.1           # ~25.5 M bf16 weights plus scale/shift
    st2, h2 = _create(sol, wk.layers, wk.in_shape, sol.BF16, sol.NET_KEEP_ACTIVATIONS)
    assert st2 == 0 and L.sol_network_workspace_bytes(h2) > 4 * ws
    L.sol_network_destroy(h)
    L.sol_network_destroy(h2)


def test_planner_rejects_bad_graphs(sol):
    bad_res = [wl.conv(8, 3), wl.conv(16, 3, res=0)]                       # residual channel mismatch
    assert _create(sol, bad_res, (1, 3, 8, 8), sol.F32)[0] == 2
    fwd_ref = [wl.conv(8, 3, src=1), wl.conv(8, 3)]                        # src must be an earlier layer
    assert _create(sol, fwd_ref, (1, 3, 8, 8), sol.F32)[0] == 2
    lin = [wl.conv(8, 3), wl.linear(4)]                                    # linear needs [n,1,1,c]
    assert _create(sol, lin, (1, 3, 8, 8), sol.F32)[0] == 6
    assert _create(sol, [wl.conv(8, 9, p=0)], (1, 3, 4, 4), sol.F32)[0] == 2   # filter larger than input
    st, h = _create(sol, wl.small_cnn_layers(), (64, 3, 32, 32), sol.F32)
    assert st == 0
    # forward without bound parameters / workspace is refused, nothing is launched
    fake = C.c_void_p(0x1000)
    assert sol.lib().sol_network_forward(h, fake, fake, fake, C.c_size_t(1 << 30), None) == 5
    sol.lib().sol_network_destroy(h)


def test_plan_tile_api_validates(sol):
    """Per-layer kernel/tile ids (set by the auto-tune, restorable by the caller) are range-checked on the host."""
    L = sol.lib()
    st, h = _create(sol, wl.small_cnn_layers(), (8, 3, 32, 32), sol.F32)
    assert st == 0
    t = C.c_int(-1)
    assert L.sol_network_layer_tile(h, 0, C.byref(t)) == 0 and t.value == 0          # heuristic until tuned
    assert L.sol_network_set_layer_tile(h, 1, 21) == 0
    assert L.sol_network_layer_tile(h, 1, C.byref(t)) == 0 and t.value == 21
    assert L.sol_network_set_layer_tile(h, 99, 21) == 2 and L.sol_network_set_layer_tile(h, 0, 1000) == 2
    assert L.sol_network_layer_tile(None, 0, C.byref(t)) == 1
    fake = C.c_void_p(0x1000)
    assert L.sol_network_autotune(None, fake, fake, fake, C.c_size_t(0), 3, None) == 1
    assert L.sol_network_autotune(h, fake, fake, fake, C.c_size_t(1 << 30), 0, None) == 2     # reps out of range
    L.sol_network_destroy(h)


def test_plan_fuses_stem_and_pool_only_when_it_may(sol):
    """The depth-first stem + max-pool pair is a plan-time decision taken on the host: bf16 7x7/2 stem with 64
    filters and ReLU whose only consumer is a 3x3/2 pad-1 max-pool layer, and no kept activations."""
    L = sol.lib()
    t = C.c_int(-1)

    def fused(layers, shape, dt, flags=0):
        st, h = _create(sol, layers, shape, dt, flags)
        assert st == 0
        r = []
        for i in range(len(layers)):
            assert L.sol_network_layer_fused_into(h, i, C.byref(t)) == 0
            r.append(t.value)
        assert L.sol_network_layer_fused_into(h, len(layers), C.byref(t)) == 2
        ws = L.sol_network_workspace_bytes(h)
        L.sol_network_destroy(h)
        return r, ws

    wk = wl.config(3)
    n = len(wk.layers)
    r, ws = fused(wk.layers, wk.in_shape, sol.BF16)
    # the pool runs inside the stem's launch; the projection shortcut of every stage's first bottleneck (a 1x1
    # convolution without activation, read only as a residual) runs inside the launch of the 1x1 convolution that adds it
    want = list(range(n))
    want[1] = 0
    shortcuts = [l["res"] for l in wk.layers if l["kind"] == "conv" and l.get("res", -1) >= 0 and wk.layers[l["res"]]["act"] == "none"]
    assert len(shortcuts) == 4 and shortcuts[0] == 4
    for j in shortcuts:
        want[j] = j + 1
    # the identity bottlenecks of stages 0 and 1 (mid widths 64 / 128, enough pixels at batch 64) run as one
    # depth-first launch: their first two convolutions are produced by the launch of the third
    ends = [i for i, l in enumerate(wk.layers) if l["kind"] == "conv" and l.get("res", -1) >= 0 and wk.layers[l["res"]]["act"] != "none"
            and l["cout"] in (256, 512)]
    assert len(ends) == 5
    for i in ends:
        want[i - 2] = want[i - 1] = i
    # the last 1x1 convolution of an identity bottleneck of stage 2 (256 -> 1024 channels at 14x14) and the first 1x1
    # convolution of the next bottleneck (1024 -> 256, and 1024 -> 512 into the last stage) run as one expand-reduce launch:
    # five pairs
    starts = [i for i, l in enumerate(wk.layers[:-1]) if l["kind"] == "conv" and l["cout"] == 1024 and l.get("res", -1) >= 0
              and wk.layers[l["res"]]["act"] != "none" and wk.layers[i + 1]["kind"] == "conv" and wk.layers[i + 1]["cout"] in (256, 512)
              and wk.layers[i + 1]["kh"] == 1]
    assert len(starts) == 5
    for i in starts:
        want[i + 1] = i
    assert r == want
    st_, h_ = _create(sol, wk.layers, wk.in_shape, sol.BF16, 0)
    bs = C.c_int(-2)
    assert [L.sol_network_layer_xr(h_, i, C.byref(bs)) or bs.value for i in starts] == [1] * 5
    assert L.sol_network_layer_xr(h_, 0, C.byref(bs)) == 0 and bs.value == -1
    assert L.sol_network_set_layer_xr(h_, starts[0], 0) == 0 and L.sol_network_layer_xr(h_, starts[0], C.byref(bs)) == 0 and bs.value == 0
    assert L.sol_network_layer_fused_into(h_, starts[0] + 1, C.byref(t)) == 0 and t.value == starts[0] + 1
    assert L.sol_network_set_layer_xr(h_, 0, 1) == 6 and L.sol_network_set_layer_xr(h_, 0, 0) == 0
    assert L.sol_network_set_layer_xr(h_, starts[0], 1) == 0
    assert [L.sol_network_layer_block(h_, i, C.byref(bs)) or bs.value for i in ends] == [1] * 5
    assert L.sol_network_layer_block(h_, 0, C.byref(bs)) == 0 and bs.value == -1
    assert L.sol_network_set_layer_block(h_, ends[0], 0) == 0 and L.sol_network_layer_block(h_, ends[0], C.byref(bs)) == 0 and bs.value == 0
    assert L.sol_network_layer_fused_into(h_, ends[0] - 1, C.byref(t)) == 0 and t.value == ends[0] - 1
    assert L.sol_network_set_layer_block(h_, 0, 1) == 6 and L.sol_network_set_layer_block(h_, 0, 0) == 0
    L.sol_network_destroy(h_)
    r_keep, ws_keep = fused(wk.layers, wk.in_shape, sol.BF16, sol.NET_KEEP_ACTIVATIONS)
    assert r_keep == list(range(n)) and ws_keep > ws
    assert fused(wk.layers, wk.in_shape, sol.BF16, sol.NET_TRAINING)[0] == list(range(n))
    assert fused(wk.layers, wk.in_shape, sol.F32)[0] == list(range(n))                     # fp32: no stem kernel
    stem, pool = wl.conv(64, 7, 2, 3), wl.pool("max", 3, 2, 1)
    tail = [wl.conv(8, 1)]
    assert fused([stem, pool] + tail, (2, 3, 40, 40), sol.BF16)[0] == [0, 0, 2]
    assert fused([stem, pool], (2, 3, 40, 40), sol.BF16)[0] == [0, 0]                      # the pool is the network output
    assert fused([stem, wl.pool("max", 2, 2, 0)] + tail, (2, 3, 40, 40), sol.BF16)[0] == [0, 1, 2]
    assert fused([stem, wl.pool("avg", 3, 2, 1)] + tail, (2, 3, 40, 40), sol.BF16)[0] == [0, 1, 2]
    assert fused([wl.conv(32, 7, 2, 3), pool] + tail, (2, 3, 40, 40), sol.BF16)[0] == [0, 1, 2]
    assert fused([wl.conv(64, 7, 2, 3, act="none"), pool] + tail, (2, 3, 40, 40), sol.BF16)[0] == [0, 1, 2]
    # a second consumer of the stem's output keeps it alive: no fusion
    assert fused([stem, pool, wl.conv(8, 1, src=0)], (2, 3, 40, 40), sol.BF16)[0] == [0, 1, 2]
    assert L.sol_network_layer_fused_into(None, 0, C.byref(t)) == 1


def test_concat_planning_and_validation(sol):
    """Channel concatenation layers: shapes, refusals, and which producers the plan lets write in place."""
    L = sol.lib()
    c, cat = wl.conv, wl.concat
    fire = wl.fire_layers(1, 0, 8, 16)
    layers = [c(16, 3)] + fire + [c(8, 1, p=0)]
    st, h = _create(sol, layers, (2, 3, 12, 12), sol.BF16)
    assert st == 0
    d = sol.TensorDesc()
    assert L.sol_network_output_desc(h, 4, C.byref(d)) == 0 and (d.n, d.h, d.w, d.c) == (2, 12, 12, 32)
    t = C.c_int(-1)
    assert L.sol_network_concat_in_place(h, 4, C.byref(t)) == 0 and t.value == 2
    assert L.sol_network_concat_in_place(h, 3, C.byref(t)) == 2            # not a concatenation
    assert L.sol_network_concat_in_place(h, 99, C.byref(t)) == 2 and L.sol_network_concat_in_place(None, 4, C.byref(t)) == 1
    ws = L.sol_network_workspace_bytes(h)
    L.sol_network_destroy(h)
    st, h = _create(sol, layers, (2, 3, 12, 12), sol.BF16, sol.NET_KEEP_ACTIVATIONS)
    assert st == 0 and L.sol_network_concat_in_place(h, 4, C.byref(t)) == 0 and t.value == 0
    assert L.sol_network_workspace_bytes(h) > ws                         # the expand outputs exist twice when everything is kept
    L.sol_network_destroy(h)
    assert _create(sol, layers, (2, 3, 12, 12), sol.BF16, sol.NET_TRAINING)[0] == 6                     # inference only
    assert _create(sol, [c(8, 3), cat(0, 0)], (1, 3, 8, 8), sol.F32)[0] == 2                            # one layer twice
    assert _create(sol, [c(8, 3), c(8, 3, s=2, src=0), cat(0, 1)], (1, 3, 8, 8), sol.F32)[0] == 2       # extents differ
    assert _create(sol, [c(8, 3), cat(0, 2), c(8, 3)], (1, 3, 8, 8), sol.F32)[0] == 2                   # names a later layer
    assert _create(sol, [cat(-1, 0)], (1, 3, 8, 8), sol.F32)[0] == 2                                    # nothing to join


def test_depthwise_planning_and_validation(sol):
    """Depthwise layers: shape inference keeps the channel count, parameters are [taps][c] + scale/shift, bad
    descriptors are refused on the host."""
    L = sol.lib()
    assert L.sol_packed_dw_weight_bytes(32, 3, 3, sol.BF16) == 32 * 9 * 2
    assert L.sol_packed_dw_weight_bytes(8, 5, 3, sol.F32) == 8 * 15 * 4 and L.sol_packed_dw_weight_bytes(0, 3, 3, sol.F32) == 0
    assert L.sol_packed_dw_weight_bytes(3, 3, 3, sol.BF16) == 64                     # 54 bytes, rounded up to 16
    wk = wl.config(6)
    st, h = _create(sol, wk.layers, wk.in_shape, sol.BF16)
    assert st == 0
    d = sol.TensorDesc()
    assert L.sol_network_output_desc(h, 1, C.byref(d)) == 0 and (d.n, d.h, d.w, d.c) == (64, 112, 112, 32)    # depthwise s1
    assert L.sol_network_output_desc(h, 3, C.byref(d)) == 0 and (d.n, d.h, d.w, d.c) == (64, 56, 56, 64)      # depthwise s2
    assert L.sol_network_output_desc(h, -1, C.byref(d)) == 0 and (d.n, d.h, d.w, d.c) == (64, 1, 1, 1000)
    # 4.2 M parameters: pointwise + classifier weights dominate, 9 values per channel for the depthwise layers
    assert 4.2e6 * 2 <= L.sol_network_param_bytes(h) <= 4.2e6 * 2 * 1.15
    L.sol_network_destroy(h)
    assert _create(sol, [wl.conv(24, 3, dw=True)], (2, 16, 8, 8), sol.BF16)[0] == 2                            # channel count must be kept
    assert _create(sol, [wl.conv(16, 3, dw=True, pool=wl.pool_desc("max", 2, 2, 0))], (2, 16, 8, 8), sol.BF16)[0] == 6
    assert _create(sol, [wl.conv(16, 3, dw=True), wl.gap(), wl.linear(4)], (2, 16, 8, 8), sol.BF16, sol.NET_TRAINING)[0] == 6
    xd = sol.TensorDesc(1, 8, 8, 16, sol.BF16)
    fake, null = C.c_void_p(0x1000), C.c_void_p(0)
    call = lambda cd, x=fake, w=fake, y=fake: L.sol_dwconv2d_fused(C.byref(xd), x, C.byref(cd), w, null, null, null, 0, y, null)  # noqa: E731
    assert call(sol.ConvDesc(32, 16, 3, 3, 1, 1, 1, 1)) == 2                          # cout != channels
    assert call(sol.ConvDesc(16, 16, 3, 3, 1, 1, 1, 1), w=null) == 1                  # NULL weights
    assert call(sol.ConvDesc(16, 16, 3, 3, 1, 1, 1, 1), x=C.c_void_p(0x1008)) == 4    # misaligned x
    assert call(sol.ConvDesc(16, 16, 11, 11, 1, 1, 0, 0)) == 2                        # filter larger than the input


def test_no_kernel_spills_registers():
    """The compiler's per-kernel resource report of the last build (written by paper_2003_10688_amd/build.py): no kernel
    of the library may use scratch memory (spilled registers travel through HBM: the stage-3 3x3 kernels once wrote
    5.7x their output that way), and none may exceed the 160 KB of LDS of a compute unit."""
    import json

    from paper_2003_10688_amd import build as b

    path = b.RESOURCES
    if not os.path.exists(path):
        pytest.skip("no build report (run __graft_entry__.build())")
    with open(path) as f:
        res = json.load(f)
    assert len(res) > 100
    spills = {k: v["scratch_bytes_per_lane"] for k, v in res.items() if v.get("scratch_bytes_per_lane", 0) != 0}
    assert not spills, spills
    assert all(v.get("lds_bytes", 0) <= 160 * 1024 for v in res.values())
