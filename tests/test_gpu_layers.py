"""GPU parity of single layers and small fused groups against the CPU oracle, through the C ABI.
Sizes span several tiles with ragged tails; forced configurations cover every register-tile
variant, streaming and resident staging, and channel slicing."""
import numpy as np
import pytest

from synth import nets, gen
from gpu_util import compare, announce

pytestmark = pytest.mark.gpu


def _mk(layers, h, w, c, dist="uniform", name="t"):
    return dict(name=name, layers=layers, in_h=h, in_w=w, in_c=c, input_dist=dist)


def _run(net, batch, seed=1, force=None, **plan):
    from oracle import oracle as o
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    x, ws, bs = gen.make_params(net, batch, seed)
    ref = o.run_net(net, x, ws, bs)
    if force is not None:
        B.dlf_debug_force_config(*force)
    try:
        s = Session(net, batch, ws, bs, **plan)
    finally:
        B.dlf_debug_force_config(0)
    try:
        got = s.run_numpy(x)
        groups = s.groups
    finally:
        s.close()
    return got, ref, groups


def _manual(n_layers, lasts, budget=64):
    from paper_2011_05630_amd import binding as B
    return dict(mode=B.TUNER_MANUAL, group_last=list(lasts), group_budget=[budget] * len(lasts))


# (th, tw, variant, nslices, slice_c, stream0)
FORCED = [
    (8, 8, 2, 1, 0, 1), (8, 8, 2, 1, 0, 0), (8, 16, 0, 1, 0, 1), (16, 16, 1, 1, 0, 1),
    (16, 16, 1, 1, 0, 0), (7, 14, 0, 1, 0, 1), (4, 28, 1, 1, 0, 1), (2, 4, 2, 1, 0, 1),
]


@pytest.mark.parametrize("force", FORCED)
def test_conv3x3_single_layer_forced_configs(force):
    announce("conv3x3 c32 37x29 b2 force", force)
    net = _mk([nets.conv(32, 64, 3, 1, 1, "relu")], 37, 29, 32)
    got, ref, _ = _run(net, 2, force=force, **_manual(1, [0]))
    compare(got, ref, "conv3x3 force=%s" % (force,))


@pytest.mark.parametrize("k", [1, 3])
@pytest.mark.parametrize("kc", [32, 64, 128])
def test_conv_streaming_round_sizes(k, kc):
    announce("conv stream round", k, kc)
    net = _mk([nets.conv(128, 96, k, 1, k // 2, "relu")], 21, 18, 128, dist="normal")
    got, ref, _ = _run(net, 2, force=(4, 8, 1, 1, 0, 1, kc), **_manual(1, [0]))
    compare(got, ref, "conv k%d stream kc=%d" % (k, kc))


@pytest.mark.parametrize("cin,cout", [(16, 16), (8, 24), (3, 32), (64, 128), (96, 40), (256, 64)])
def test_conv3x3_channel_shapes(cin, cout):
    announce("conv3x3 channels", cin, cout)
    net = _mk([nets.conv(cin, cout, 3, 1, 1, "relu")], 19, 23, cin)
    got, ref, _ = _run(net, 3, **_manual(1, [0]))
    compare(got, ref, "conv3x3 %d->%d" % (cin, cout))


@pytest.mark.parametrize("k,stride,pad,cin,cout,hw", [
    (1, 1, 0, 64, 256, 28), (1, 2, 0, 64, 128, 28), (3, 2, 1, 32, 32, 29), (7, 2, 3, 3, 64, 50),
    (5, 1, 2, 16, 32, 17), (11, 4, 2, 3, 64, 67), (3, 1, 0, 16, 16, 12)])
def test_conv_kernel_stride_pad(k, stride, pad, cin, cout, hw):
    announce("conv k/s/p", k, stride, pad, cin, cout, hw)
    net = _mk([nets.conv(cin, cout, k, stride, pad, "relu")], hw, hw + 3, cin, dist="normal")
    got, ref, _ = _run(net, 2, **_manual(1, [0]))
    compare(got, ref, "conv k%d s%d p%d" % (k, stride, pad))


@pytest.mark.parametrize("k,stride,pad,cin,cout,hw", [
    (3, 2, 1, 3, 32, 33), (7, 2, 3, 3, 64, 61), (5, 2, 2, 4, 16, 30), (3, 2, 1, 1, 8, 21),
    (11, 4, 2, 3, 64, 67), (3, 4, 0, 2, 32, 40), (7, 2, 3, 3, 64, 224)])
def test_narrow_input_even_stride(k, stride, pad, cin, cout, hw):
    """cin <= 4 with an even stride: filter columns folded into the channel dimension."""
    announce("narrow conv", k, stride, pad, cin, cout, hw)
    net = _mk([nets.conv(cin, cout, k, stride, pad, "relu")], hw, hw + 5, cin, dist="normal")
    got, ref, _ = _run(net, 2, **_manual(1, [0]))
    compare(got, ref, "narrow conv k%d s%d cin%d" % (k, stride, cin))
    for force in ((4, 8, 2, 1, 0, 0), (7, 14, 0, 1, 0, 0), (8, 16, 1, 1, 0, 0)):
        got, ref, _ = _run(net, 2, force=force, **_manual(1, [0]))
        compare(got, ref, "narrow conv k%d s%d cin%d force %s" % (k, stride, cin, force))


def test_narrow_input_stems_fused():
    announce("fused stems")
    layers = [nets.conv(3, 64, 7, 2, 3, "relu"), nets.maxpool(64, 3, 2, 1)]
    net = _mk(layers, 99, 83, 3, dist="normal")
    got, ref, g = _run(net, 2, **_manual(2, [1]))
    assert len(g) == 1
    compare(got, ref, "7x7 s2 stem + 3x3 s2 pool")
    layers = [nets.conv(3, 32, 3, 2, 1, "relu6"), nets.dwconv(32, 3, 1, "relu6"),
              nets.conv(32, 64, 1, 1, 0, "relu6"), nets.dwconv(64, 3, 2, "relu6")]
    net = _mk(layers, 64, 72, 3, dist="normal")
    got, ref, g = _run(net, 2, **_manual(4, [3]))
    assert len(g) == 1
    compare(got, ref, "3x3 s2 stem + dw + pw + dw s2")


@pytest.mark.parametrize("k,stride,pad,cin,mid,pool,h,w", [
    (3, 1, 1, 3, 64, True, 38, 50),     # K = 27 -> 32: 4 parts per row (divides the workgroup)
    (3, 1, 1, 5, 32, False, 21, 35),    # K = 45 -> 64: 8 parts per row, odd channel count
    (5, 1, 2, 3, 32, False, 29, 23),    # K = 75 -> 96: 12 parts per row (does not divide it)
    (7, 1, 3, 3, 32, True, 30, 26),     # K = 147 -> 160: 20 parts per row
    (3, 3, 0, 3, 32, False, 40, 31),    # odd stride, no padding
    (3, 1, 1, 1, 16, False, 19, 19),    # one input channel
])
def test_narrow_input_gathered_through_lds(k, stride, pad, cin, mid, pool, h, w):
    """A narrow first layer that is not folded by rows (odd stride or more than 4 channels), fused
    with a second convolution: the image patch goes through a spare LDS area and the im2col rows
    are copied out of it.  Tiles forced small enough that borders, ragged tiles and several tiles
    per image occur; the automatic choice as well."""
    announce("narrow gathered", k, stride, pad, cin, mid, pool, h, w)
    layers = [nets.conv(cin, mid, k, stride, pad, "relu"), nets.conv(mid, 32, 3, 1, 1, "relu")]
    if pool:
        layers.append(nets.maxpool(32, 2, 2, 0))
    net = _mk(layers, h, w, cin, dist="normal")
    last = len(layers) - 1
    got, ref, g = _run(net, 2, **_manual(len(layers), [last]))
    assert len(g) == 1
    compare(got, ref, "narrow gathered k%d s%d cin%d" % (k, stride, cin))
    for force in ((4, 8, 2, 1, 0, 0), (2, 16, 3, 1, 0, 0), (5, 6, 0, 1, 0, 0)):
        got, ref, g = _run(net, 2, force=force, **_manual(len(layers), [last]))
        assert len(g) == 1
        compare(got, ref, "narrow gathered k%d s%d cin%d force %s" % (k, stride, cin, force))


@pytest.mark.parametrize("slices", [(8, 8, 0, 4, 64, 1), (8, 8, 1, 2, 128, 1), (7, 7, 0, 2, 128, 1),
                                    (8, 8, 2, 8, 32, 1), (8, 8, 1, 4, 64, 1, 64)])
def test_conv_output_channel_slices(slices):
    announce("conv slices", slices)
    net = _mk([nets.conv(64, 256, 3, 1, 1, "relu")], 14, 14, 64)
    got, ref, _ = _run(net, 2, force=slices, **_manual(1, [0]))
    compare(got, ref, "conv slices %s" % (slices,))


@pytest.mark.parametrize("cin,cout,hw,stride,act,batch", [
    (64, 256, 28, 1, "relu", 2), (256, 64, 28, 1, "relu", 2), (32, 64, 33, 1, "relu6", 3),
    (256, 512, 28, 2, "none", 2), (96, 40, 7, 1, "relu", 3), (64, 8, 9, 1, "relu", 1),
    (1024, 256, 14, 1, "relu", 5), (128, 128, 15, 2, "relu6", 2), (32, 1000, 3, 1, "none", 7),
    (2048, 512, 7, 1, "relu", 3), (512, 40, 7, 2, "relu", 2)])
def test_pointwise_kernel(cin, cout, hw, stride, act, batch):
    """1x1 convolutions on the barrier-free pointwise kernel (forced), ragged pixel and channel
    counts included."""
    announce("pointwise", cin, cout, hw, stride, act, batch)
    from paper_2011_05630_amd import binding as B
    net = _mk([nets.conv(cin, cout, 1, stride, 0, act)], hw, hw + 2, cin, dist="normal")
    for mode in (3, 4, 5, 6, 7):      # 64x64, 32x32, split-K 64x64 items; 128x128 and 64x256 blocks
        B.dlf_debug_pointwise_mode(mode)
        try:
            got, ref, g = _run(net, batch, **_manual(1, [0]))
        finally:
            B.dlf_debug_pointwise_mode(0)
        compare(got, ref, "pointwise %d->%d s%d shape %d" % (cin, cout, stride, mode - 3))


def test_pointwise_kernel_is_used_and_adds_residual():
    announce("pointwise residual")
    from oracle import oracle as o
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    layers = [nets.conv(64, 64, 3, 1, 1, "relu"), nets.conv(64, 256, 1, 1, 0, "relu"),
              nets.conv(256, 64, 1, 1, 0, "relu"), nets.conv(64, 256, 1, 1, 0, "relu", residual_from=1)]
    net = _mk(layers, 21, 19, 64, dist="normal")
    x, ws, bs = gen.make_params(net, 3)
    ref = o.run_net(net, x, ws, bs)
    for mode in (1, 3, 4, 5, 6, 7):
        B.dlf_debug_pointwise_mode(mode)
        try:
            s = Session(net, 3, ws, bs, **_manual(4, [0, 1, 2, 3]))
        finally:
            B.dlf_debug_pointwise_mode(0)
        try:
            kinds = [B.dlf_plan_group_config(s.plan, i)["kind"] for i in range(4)]
            got = s.run_numpy(x)
        finally:
            s.close()
        assert kinds == [0, 3, 3, 3], kinds
        compare(got, ref, "pointwise chain with residual, mode %d" % mode)
    # never mode: same result from the fused-group kernel
    B.dlf_debug_pointwise_mode(2)
    try:
        s = Session(net, 3, ws, bs, **_manual(4, [0, 1, 2, 3]))
    finally:
        B.dlf_debug_pointwise_mode(0)
    try:
        kinds = [B.dlf_plan_group_config(s.plan, i)["kind"] for i in range(4)]
        got2 = s.run_numpy(x)
    finally:
        s.close()
    assert kinds == [0, 0, 0, 0], kinds
    compare(got2, ref, "same chain, fused-group kernel")


def test_pointwise_split_k_with_residual():
    announce("pointwise split-K residual")
    from paper_2011_05630_amd import binding as B
    layers = [nets.conv(512, 256, 1, 1, 0, "relu"), nets.conv(256, 256, 1, 1, 0, "relu6"),
              nets.conv(256, 256, 1, 1, 0, "relu", residual_from=0)]
    net = _mk(layers, 9, 11, 512, dist="normal")
    B.dlf_debug_pointwise_mode(5)
    try:
        got, ref, g = _run(net, 3, **_manual(3, [0, 1, 2]))
    finally:
        B.dlf_debug_pointwise_mode(0)
    compare(got, ref, "split-K pointwise chain with residual")


@pytest.mark.parametrize("act", ["none", "relu", "relu6"])
def test_activations_and_bias(act):
    announce("act", act)
    net = _mk([nets.conv(16, 16, 3, 1, 1, act)], 9, 9, 16, dist="normal")
    x, ws, bs = gen.make_params(net, 1)
    got, ref, _ = _run(net, 1, **_manual(1, [0]))
    compare(got, ref, "act " + act)
    if act == "relu6":
        assert got.max() <= 6.0 and got.min() >= 0.0


def test_residual_add_from_hbm():
    announce("residual")
    layers = [nets.conv(32, 32, 3, 1, 1, "relu"), nets.conv(32, 32, 3, 1, 1, "relu"),
              nets.conv(32, 32, 1, 1, 0, "relu", residual_from=0)]
    net = _mk(layers, 20, 20, 32)
    got, ref, _ = _run(net, 2, **_manual(3, [0, 1, 2]))
    compare(got, ref, "residual unfused")
    got, ref, _ = _run(net, 2, **_manual(3, [0, 2]))
    compare(got, ref, "residual, layers 1-2 fused")


@pytest.mark.parametrize("k,stride,pad,hw", [(2, 2, 0, 16), (3, 2, 1, 17), (3, 2, 0, 15),
                                             (2, 2, 0, 15)])
def test_maxpool_standalone(k, stride, pad, hw):
    announce("maxpool", k, stride, pad, hw)
    # negative inputs: a zero pad would win, -inf padding must not
    net = _mk([nets.maxpool(64, k, stride, pad)], hw, hw + 2, 64, dist="normal")
    from oracle import oracle as o
    from paper_2011_05630_amd.runner import Session
    x, ws, bs = gen.make_params(net, 2)
    x = (x - np.float16(3.0)).astype(np.float16)
    ref = o.run_net(net, x, ws, bs)
    s = Session(net, 2, ws, bs)
    got = s.run_numpy(x)
    s.close()
    assert np.array_equal(got.astype(np.float32), ref)   # pooling is exact


def test_conv_with_fused_pool2():
    announce("conv+pool2 fused")
    layers = [nets.conv(16, 32, 3, 1, 1, "relu"), nets.maxpool(32, 2, 2, 0)]
    net = _mk(layers, 24, 20, 16)
    got, ref, g = _run(net, 2, **_manual(2, [1]))
    assert len(g) == 1
    compare(got, ref, "conv+pool fused")
    got, ref, g = _run(net, 2, **_manual(2, [0, 1]))
    compare(got, ref, "conv, pool separate")
    # sliced over output channels
    layers = [nets.conv(32, 128, 3, 1, 1, "relu"), nets.maxpool(128, 2, 2, 0)]
    net = _mk(layers, 16, 16, 32)
    got, ref, g = _run(net, 1, force=(4, 4, 0, 2, 64, 1), **_manual(2, [1]))
    compare(got, ref, "conv+pool fused, 2 slices")


@pytest.mark.parametrize("stride,c,hw", [(1, 32, 20), (2, 64, 21), (1, 128, 9), (2, 8, 12)])
def test_depthwise(stride, c, hw):
    announce("depthwise", stride, c, hw)
    net = _mk([nets.dwconv(c, 3, stride, "relu6")], hw, hw + 1, c, dist="normal")
    got, ref, _ = _run(net, 2)
    compare(got, ref, "dw s%d c%d" % (stride, c))


def _run_dw_mode(net, batch, mode, seed=1, **plan):
    """_run with the planner's choice between the fused-group kernel and the streaming depthwise
    kernels fixed (1 = streaming wherever it applies, 2 = never)."""
    from paper_2011_05630_amd import binding as B
    B.dlf_debug_depthwise_mode(mode)
    try:
        return _run(net, batch, seed=seed, **plan)
    finally:
        B.dlf_debug_depthwise_mode(0)


# (stride, channels, height, width, batch, activation): maps of one strip and of several with a ragged
# last one, widths whose rows are not whole runs of 64 vectors, 8 to 1024 channels (one to 128 vectors
# per pixel), odd and even sizes under stride 2, one-pixel-wide and one-row maps
DW_CASES = [(1, 32, 20, 21, 2, "relu6"), (2, 64, 21, 22, 2, "relu6"), (1, 128, 9, 10, 2, "relu6"),
            (2, 8, 12, 13, 2, "none"), (1, 8, 31, 5, 3, "relu"), (1, 24, 30, 17, 1, "relu6"),
            (2, 40, 29, 30, 2, "relu6"), (1, 512, 14, 14, 3, "relu6"), (2, 512, 14, 14, 2, "relu6"),
            (1, 1024, 7, 7, 2, "relu6"), (1, 16, 1, 9, 2, "none"), (1, 16, 9, 1, 2, "relu"),
            (2, 16, 2, 2, 1, "relu"), (1, 64, 57, 56, 1, "relu6"), (2, 32, 112, 112, 1, "relu6")]


@pytest.mark.parametrize("stride,c,h,w,batch,act", DW_CASES)
def test_depthwise_streaming_kernel(stride, c, h, w, batch, act):
    from paper_2011_05630_amd import binding as B
    announce("depthwise streaming", stride, c, h, w, batch, act)
    net = _mk([nets.dwconv(c, 3, stride, act)], h, w, c, dist="normal")
    B.dlf_debug_depthwise_mode(1)
    try:
        from paper_2011_05630_amd.runner import Session
        from oracle import oracle as o
        x, ws, bs = gen.make_params(net, batch, 7)
        s = Session(net, batch, ws, bs)
    finally:
        B.dlf_debug_depthwise_mode(0)
    try:
        cfg = B.dlf_plan_group_config(s.plan, 0)
        assert cfg["kind"] == 5 and cfg["variant"] == stride - 1, cfg
        got = s.run_numpy(x)
    finally:
        s.close()
    compare(got, o.run_net(net, x, ws, bs), "dw stream s%d c%d %dx%d" % (stride, c, h, w))


def test_depthwise_streaming_kernel_equals_fused_group_kernel():
    """The two kernels accumulate the nine taps in the same order in fp32 and round once: same bits."""
    net = _mk([nets.dwconv(64, 3, 1, "relu6")], 33, 29, 64, dist="normal")
    a, ref, _ = _run_dw_mode(net, 2, 1)
    b, _, _ = _run_dw_mode(net, 2, 2)
    compare(a, ref, "dw streaming")
    compare(b, ref, "dw in the fused-group kernel")
    assert np.array_equal(a, b)


# (stride, channels in, channels out, height, width, batch): 2 or 4 channel blocks per work item and
# several channel groups, a ragged last pixel group, maps narrower than a pixel group (rows wrap
# inside a group), images that end inside a group, one pixel
DWPW_CASES = [(1, 32, 64, 28, 28, 2), (2, 64, 128, 21, 23, 2), (1, 128, 128, 9, 10, 3), (2, 128, 256, 14, 14, 2),
              (1, 256, 512, 7, 7, 3), (1, 512, 512, 14, 14, 2), (1, 32, 24, 13, 5, 1), (1, 64, 200, 6, 9, 2),
              (2, 32, 64, 1, 1, 3), (1, 1024, 1024, 7, 7, 1), (2, 32, 64, 112, 112, 1)]


@pytest.mark.parametrize("stride,c,cout,h,w,batch", DWPW_CASES)
def test_depthwise_pointwise_fused_kernel(stride, c, cout, h, w, batch):
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    from oracle import oracle as o
    announce("dw+pw fused kernel", stride, c, cout, h, w, batch)
    layers = [nets.dwconv(c, 3, stride, "relu6"), nets.conv(c, cout, 1, 1, 0, "relu6" if cout != 24 else "none")]
    net = _mk(layers, h, w, c, dist="normal")
    x, ws, bs = gen.make_params(net, batch, 9)
    B.dlf_debug_depthwise_mode(3)
    try:
        s = Session(net, batch, ws, bs, **_manual(2, [1]))
    finally:
        B.dlf_debug_depthwise_mode(0)
    try:
        cfg = B.dlf_plan_group_config(s.plan, 0)
        assert len(s.groups) == 1 and cfg["kind"] == 6 and cfg["variant"] in (2, 4), cfg
        got = s.run_numpy(x)
    finally:
        s.close()
    compare(got, o.run_net(net, x, ws, bs), "dw+pw s%d %d->%d %dx%d" % (stride, c, cout, h, w))


# (stride, channels in, channels out, height, width, batch, channel blocks per wave, channels per pass;
# 0, 0 = the planner's choice): the kernel for maps of many channels and few pixels: one and several
# passes over the channels (256 .. 1024 in passes of 256 or 512) with all regions resident or one at
# a time, both strides, one and two channel blocks per wave, several slices of the output channels
# and a ragged last one, waves without a channel block, maps cut into several tiles with the last
# row / column of tiles overhanging, tiles of fewer than 32 pixels, one-pixel maps, odd sizes under
# stride 2
DWS_CASES = [(1, 512, 512, 14, 14, 3, 2, 512), (1, 512, 512, 14, 14, 2, 1, 256), (1, 256, 256, 7, 7, 2, 0, 0),
             (2, 256, 512, 28, 28, 2, 2, 256), (2, 512, 1024, 14, 14, 2, 0, 0), (2, 512, 1024, 14, 14, 1, 2, 256),
             (1, 1024, 1024, 7, 7, 2, 2, 512), (1, 1024, 1024, 7, 7, 2, 1, 256), (1, 768, 200, 9, 11, 2, 0, 0),
             (1, 512, 96, 3, 5, 3, 1, 512), (2, 512, 640, 13, 11, 1, 2, 256), (1, 256, 1024, 1, 1, 4, 2, 256),
             (2, 256, 64, 2, 2, 2, 0, 0), (1, 512, 512, 17, 8, 1, 2, 256), (2, 1024, 256, 9, 9, 2, 1, 256),
             (2, 1024, 512, 9, 11, 1, 2, 256), (1, 1024, 320, 8, 8, 2, 2, 256)]


@pytest.mark.parametrize("stride,c,cout,h,w,batch,cbw,kh", DWS_CASES)
def test_depthwise_pointwise_small_map_kernel(stride, c, cout, h, w, batch, cbw, kh):
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    from oracle import oracle as o
    announce("dw+pw small-map kernel", stride, c, cout, h, w, batch, cbw, kh)
    layers = [nets.dwconv(c, 3, stride, "relu6"), nets.conv(c, cout, 1, 1, 0, "relu6" if cout != 200 else "none")]
    net = _mk(layers, h, w, c, dist="normal")
    x, ws, bs = gen.make_params(net, batch, 11)
    B.dlf_debug_depthwise_mode(4)
    B.dlf_debug_depthwise_tile(cbw, kh)       # under mode 4: channel blocks per wave, channels per pass
    try:
        s = Session(net, batch, ws, bs, **_manual(2, [1]))
    finally:
        B.dlf_debug_depthwise_mode(0)
        B.dlf_debug_depthwise_tile(0, 0)
    try:
        cfg = B.dlf_plan_group_config(s.plan, 0)
        assert len(s.groups) == 1 and cfg["kind"] == 9 and cfg["variant"] // 2 == stride - 1, cfg
        if cbw:
            assert cfg["variant"] % 2 == cbw - 1, cfg
        got = s.run_numpy(x)
    finally:
        s.close()
    compare(got, o.run_net(net, x, ws, bs), "dw+pw small map s%d %d->%d %dx%d" % (stride, c, cout, h, w))


# (stride, channels in, channels out, height, width, batch, waves along x, rows per wave; 0, 0 = the
# planner's choice): every power-of-two channel count the kernel takes, tiles that overhang the map
# on both sides, one to eight pixel blocks per tile, 1 to 32 channel blocks, more and fewer work
# units than waves
DWT_CASES = [(1, 32, 64, 28, 28, 2, 0, 0), (1, 32, 64, 30, 37, 2, 2, 4), (1, 32, 64, 9, 70, 1, 4, 1),
             (2, 64, 128, 21, 23, 2, 0, 0), (2, 64, 128, 33, 31, 1, 4, 8), (1, 64, 24, 13, 5, 3, 1, 2),
             (1, 128, 128, 9, 10, 3, 0, 0), (1, 128, 128, 20, 20, 2, 4, 16), (2, 128, 256, 14, 14, 2, 2, 7),
             (1, 256, 512, 7, 7, 3, 0, 0), (1, 256, 256, 28, 28, 2, 4, 14), (1, 512, 512, 14, 14, 2, 0, 0),
             (2, 512, 1024, 14, 14, 2, 4, 7), (1, 512, 200, 6, 9, 2, 2, 2), (2, 32, 64, 1, 1, 3, 0, 0),
             (2, 32, 64, 112, 112, 1, 0, 0)]


@pytest.mark.parametrize("stride,c,cout,h,w,batch,wx,rw", DWT_CASES)
def test_depthwise_pointwise_tile_kernel(stride, c, cout, h, w, batch, wx, rw):
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    from oracle import oracle as o
    announce("dw+pw tile kernel", stride, c, cout, h, w, batch, wx, rw)
    layers = [nets.dwconv(c, 3, stride, "relu6"), nets.conv(c, cout, 1, 1, 0, "relu6" if cout != 24 else "none")]
    net = _mk(layers, h, w, c, dist="normal")
    x, ws, bs = gen.make_params(net, batch, 10)
    B.dlf_debug_depthwise_mode(1)
    B.dlf_debug_depthwise_tile(wx, rw)
    try:
        s = Session(net, batch, ws, bs, **_manual(2, [1]))
    finally:
        B.dlf_debug_depthwise_mode(0)
        B.dlf_debug_depthwise_tile(0, 0)
    try:
        cfg = B.dlf_plan_group_config(s.plan, 0)
        assert len(s.groups) == 1 and cfg["kind"] == 7 and cfg["variant"] == stride - 1, cfg
        if wx:
            assert (s.groups[0]["tile_h"], s.groups[0]["tile_w"]) == ((4 // wx) * rw, wx * 512 // c)
        got = s.run_numpy(x)
    finally:
        s.close()
    compare(got, o.run_net(net, x, ws, bs), "dw+pw tile s%d %d->%d %dx%d" % (stride, c, cout, h, w))


def test_depthwise_channel_slices():
    announce("depthwise slices")
    net = _mk([nets.dwconv(128, 3, 1, "relu6")], 14, 14, 128, dist="normal")
    got, ref, _ = _run(net, 2, force=(7, 7, 0, 4, 32, 0))
    compare(got, ref, "dw 4 slices")


def test_dw_pw_fused_and_unfused():
    announce("dw+pw")
    layers = [nets.dwconv(32, 3, 1, "relu6"), nets.conv(32, 64, 1, 1, 0, "relu6")]
    net = _mk(layers, 28, 28, 32, dist="normal")
    got, ref, g = _run(net, 2, **_manual(2, [1]))
    assert len(g) == 1
    compare(got, ref, "dw+pw fused")
    got, ref, g = _run(net, 2, **_manual(2, [0, 1]))
    compare(got, ref, "dw, pw separate")


@pytest.mark.parametrize("stride,cin,width,hw,batch", [(1, 64, 64, 28, 2), (2, 256, 128, 28, 3), (2, 64, 32, 15, 2),
                                                     (1, 32, 32, 9, 5), (2, 512, 256, 14, 2)])
def test_projection_shortcut_fused_into_the_last_pointwise_layer(stride, cin, width, hw, batch):
    """A bottleneck block with a projection shortcut: the projection and the block's last 1x1 layer
    as one group whose K loop runs over both operand pairs (kind 8), against the same block with the
    projection written to memory and added as a residual."""
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    from oracle import oracle as o
    announce("projection + 1x1", stride, cin, width, hw, batch)
    cout = 4 * width
    layers = [nets.conv(cin, width, 1, 1, 0, "relu"), nets.conv(width, width, 3, stride, 1, "relu"),
              nets.conv(cin, cout, 1, stride, 0, "none", input_from=-1),
              nets.conv(width, cout, 1, 1, 0, "relu", input_from=1, residual_from=2)]
    layers[2]["input_from"] = -1
    net = _mk([nets.conv(cin, cin, 1, 1, 0, "relu")] + [dict(L) for L in layers], hw, hw + 1, cin, dist="normal")
    # indices shift by one: the block reads layer 0
    net["layers"][3]["input_from"] = 0
    net["layers"][4]["input_from"] = 2
    net["layers"][4]["residual_from"] = 3
    x, ws, bs = gen.make_params(net, batch, 12, residual_gain=1.0)
    ref = o.run_net(net, x, ws, bs)
    outs = {}
    for name, lasts, mode in (("fused", [0, 1, 2, 4], 1), ("separate", [0, 1, 2, 3, 4], 2)):
        B.dlf_debug_pointwise_mode(mode)
        try:
            s = Session(net, batch, ws, bs, **_manual(5, lasts))
        finally:
            B.dlf_debug_pointwise_mode(0)
        try:
            kinds = [B.dlf_plan_group_config(s.plan, g)["kind"] for g in range(len(s.groups))]
            assert (kinds[-1] == 8) == (name == "fused"), kinds
            if name == "fused":
                assert B.dlf_plan_group_io(s.plan, len(s.groups) - 1) == (2, 0)
            outs[name] = s.run_numpy(x)
        finally:
            s.close()
        compare(outs[name], ref, "projection %s" % name)


def test_fc_and_global_avgpool():
    announce("gap + fc")
    layers = [nets.conv(16, 64, 3, 1, 1, "relu"), nets.gavgpool(64), nets.fc(64, 1000, "none")]
    net = _mk(layers, 7, 7, 16)
    got, ref, _ = _run(net, 5)
    compare(got, ref, "conv-gap-fc")
    layers = [nets.fc(7 * 7 * 32, 200, "relu"), nets.fc(200, 40, "none")]
    net = _mk(layers, 7, 7, 32)
    got, ref, _ = _run(net, 37)          # batch above 32: two passes in the FC kernel
    compare(got, ref, "fc-fc batch 37")


def test_fc_long_ragged_k_in_one_workgroup():
    """K = 2056: 129 K steps, so each wave's operand ring turns without tests before its last
    turns, and the last step is half beyond K (its activation vector is read from a stand-in
    address and replaced by zero).  K slices forced to 1: the plain kernel, not the split one."""
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    from oracle import oracle as o
    announce("fc K=2056, one slice")
    net = _mk([nets.fc(2056, 72, "relu")], 1, 1, 2056, dist="normal")
    x, ws, bs = gen.make_params(net, 5)
    B.dlf_debug_force_config(1, 1, 0, 1, 0, 0, 32)
    try:
        s = Session(net, 5, ws, bs)
    finally:
        B.dlf_debug_force_config(0, 0, 0, 1, 0, 0, 32)
    try:
        assert B.dlf_plan_group_config(s.plan, 0)["kind"] == 1
        assert B.dlf_plan_workspace_bytes(s.plan) == 0, "no partial sums: K is not split"
        got = s.run_numpy(x)
    finally:
        s.close()
    compare(got, o.run_net(net, x, ws, bs), "fc K=2056")


@pytest.mark.parametrize("cin,cout,hw,ks,tile,var,nsl,sc,kh,stride,act", [
    (256, 64, 7, 4, (7, 7), 2, 1, 0, 3, 1, "relu"),      # two work items x 4 K slices
    (512, 128, 7, 8, (7, 7), 2, 4, 32, 3, 1, "relu"),    # sliced channels, one item x 8
    (128, 96, 14, 2, (4, 14), 3, 1, 0, 3, 1, "relu6"),   # 128-register build, ragged channel blocks
    (256, 40, 9, 4, (4, 8), 2, 1, 0, 3, 2, "none"),      # stride 2, ragged tiles and channels
    (512, 64, 5, 8, (7, 7), 2, 2, 32, 1, 1, "relu"),     # 1x1 filter, tile larger than the map
    (64, 64, 8, 2, (8, 8), 2, 1, 0, 5, 1, "relu"),       # 5x5 filter (generic tap loop)
])
def test_conv_k_split_over_waves(cin, cout, hw, ks, tile, var, nsl, sc, kh, stride, act):
    """A single resident convolution whose K is split over the waves of a workgroup (partial sums
    through LDS), forced.  The form exists for one-stage groups only."""
    announce("conv ksplit", cin, cout, hw, ks, tile, var, nsl, sc, kh, stride, act)
    from oracle import oracle as o
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    nets_ = [_mk([nets.conv(cin, cout, kh, stride, kh // 2, act)], hw, hw + 1, cin, dist="normal")]
    for net in nets_:
        x, ws, bs = gen.make_params(net, 3)
        ref = o.run_net(net, x, ws, bs)
        B.dlf_debug_force_config(tile[0], tile[1], var, nsl, sc, 0, 32)
        B.dlf_debug_force_ksplit(ks)
        try:
            s = Session(net, 3, ws, bs, **_manual(len(net["layers"]), [len(net["layers"]) - 1]))
        finally:
            B.dlf_debug_force_config(0)
        try:
            got = s.run_numpy(x)
        finally:
            s.close()
        compare(got, ref, "conv %d->%d k%d s%d, K over %d waves" % (cin, cout, kh, stride, ks))


@pytest.mark.parametrize("cin,cout,h,w,batch,shape,th,tw,pool,act,res", [
    (64, 128, 20, 24, 2, 1, 8, 28, 0, "relu", 0),      # ragged tiles in both directions, one activation block
    (32, 64, 16, 16, 1, 2, 16, 32, 0, "none", 0),      # tile wider than the map, two weight stages only
    (128, 72, 14, 14, 3, 0, 14, 16, 0, "relu6", 0),    # ragged channel group, 196 of 256 pixels
    (64, 64, 12, 12, 2, 3, 8, 8, 1, "relu", 0),        # folded 2x2 pool, small tiles
    (96, 200, 28, 28, 2, 0, 8, 28, 1, "relu", 0),      # folded pool, ragged channels and rows, three blocks
    (64, 64, 30, 30, 2, 1, 16, 16, 0, "relu", 1),      # residual operand
    (256, 256, 14, 14, 2, 2, 14, 32, 0, "relu", 1),    # long K: ring and buffers wrap many times
    (256, 128, 14, 14, 2, 1, 8, 28, 0, "relu", 0),     # 64-channel blocks, four of them, two-stage ring
    (192, 64, 9, 9, 1, 3, 4, 14, 0, "relu", 0),        # 64-channel blocks, three of them
    (32, 32, 5, 5, 1, 0, 2, 4, 0, "relu", 0),          # tiny tiles: one activation load per block
    (64, 160, 40, 36, 2, 4, 16, 32, 0, "relu", 0),     # 128 x 512 blocks: ragged tiles and channel groups
    (128, 128, 32, 32, 1, 4, 16, 32, 1, "relu6", 0),   # 128 x 512 blocks with the folded pool
    (64, 64, 30, 30, 2, 4, 14, 28, 0, "relu", 1),      # 128 x 512 blocks, 392 pixels, residual, half the channels
])
def test_block3x3_kernel(cin, cout, h, w, batch, shape, th, tw, pool, act, res):
    """The block 3x3 kernel, forced with a given shape, against the layer-by-layer oracle."""
    announce("block 3x3", cin, cout, h, w, batch, shape, th, tw, pool, act, res)
    from oracle import oracle as o
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    layers = []
    if res:
        layers.append(nets.conv(cin, cout, 1, 1, 0, "relu"))
        layers.append(nets.conv(cout, cout, 3, 1, 1, act, residual_from=0))
        lasts = [0, 1]
    else:
        layers.append(nets.conv(cin, cout, 3, 1, 1, act))
        lasts = [0]
        if pool:
            layers.append(nets.maxpool(cout, 2, 2, 0))
            lasts = [1]
    net = _mk(layers, h, w, cin, dist="normal")
    x, ws, bs = gen.make_params(net, batch, 5)
    ref = o.run_net(net, x, ws, bs)
    B.dlf_debug_block3x3_mode(1, shape, th, tw)
    try:
        s = Session(net, batch, ws, bs, **_manual(len(layers), lasts))
    finally:
        B.dlf_debug_block3x3_mode(0)
    try:
        cfg = B.dlf_plan_group_config(s.plan, len(lasts) - 1)
        assert cfg["kind"] == 4 and cfg["variant"] == shape, "the block 3x3 kernel must be the one that runs"
        got = s.run_numpy(x)
    finally:
        s.close()
    compare(got, ref, "block 3x3 %d->%d %dx%d shape %d tile %dx%d" % (cin, cout, h, w, shape, th, tw))


# (channels in, channels out, height, width, batch, waves per channel block (0 = the planner's choice),
# activation): the 3x3 kernel for maps of many channels and few pixels: 32, 64 and 128 sixteen-byte
# parts per pixel, K whole or split over 2 or 4 waves, several slices of the output channels and a
# ragged last one, waves without a channel block, maps of one tile and of several with the last row /
# column of tiles overhanging, tiles of fewer than 32 pixels, a one-pixel map
C3S_CASES = [(256, 256, 14, 14, 2, 2, "relu", 1), (256, 256, 14, 14, 3, 1, "relu", 1), (512, 512, 7, 7, 2, 4, "relu", 1),
             (512, 512, 14, 14, 1, 2, "relu6", 1), (1024, 256, 5, 6, 2, 1, "relu", 1), (256, 200, 9, 11, 2, 4, "none", 1),
             (512, 96, 3, 5, 3, 2, "relu", 1), (256, 1024, 1, 1, 4, 0, "relu", 1), (512, 640, 17, 8, 1, 0, "relu", 1),
             (256, 64, 7, 7, 4, 0, "relu", 1), (1024, 1024, 4, 4, 1, 4, "relu", 1),
             # stride 2: even and odd maps, regions that only fit LDS for smaller tiles (the planner's cut), one
             # 32-pixel block per tile, a map that shrinks to one pixel
             (256, 256, 28, 28, 2, 0, "relu", 2), (512, 512, 14, 14, 2, 0, "relu", 2), (256, 96, 13, 15, 2, 2, "relu6", 2),
             (1024, 128, 9, 7, 1, 0, "relu", 2), (256, 64, 2, 2, 3, 4, "none", 2), (2048, 64, 6, 6, 1, 0, "relu", 1)]


@pytest.mark.parametrize("cin,cout,h,w,batch,ksplit,act,stride", C3S_CASES)
def test_small_map_3x3_kernel(cin, cout, h, w, batch, ksplit, act, stride):
    from oracle import oracle as o
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    announce("small-map 3x3", cin, cout, h, w, batch, ksplit, act, stride)
    net = _mk([nets.conv(cin, cout, 3, stride, 1, act)], h, w, cin, dist="normal")
    x, ws, bs = gen.make_params(net, batch, 12)
    B.dlf_debug_block3x3_mode(1, 5, ksplit, 0)        # shape 5: this kernel; th = waves per channel block
    try:
        s = Session(net, batch, ws, bs, **_manual(1, [0]))
    finally:
        B.dlf_debug_block3x3_mode(0)
    try:
        cfg = B.dlf_plan_group_config(s.plan, 0)
        assert cfg["kind"] == 10, cfg
        if ksplit:
            assert cfg["variant"] == ksplit, cfg
        got = s.run_numpy(x)
    finally:
        s.close()
    compare(got, o.run_net(net, x, ws, bs), "small-map 3x3 s%d %d->%d %dx%d" % (stride, cin, cout, h, w))


# (cin, cout, height, width, batch, waves per channel block, activation, stride): the same kernel with a residual
# operand added before the activation (the second 3x3 layer of a basic residual block): one and two 32-pixel
# blocks, K shared by 1, 2 and 4 waves, a ragged last channel block, ragged tiles, stride 2
C3S_RES_CASES = [(256, 256, 14, 14, 2, 2, "relu", 1), (512, 512, 7, 7, 3, 4, "relu", 1), (256, 200, 9, 11, 2, 1, "relu6", 1),
                 (512, 96, 3, 5, 3, 0, "none", 1), (256, 256, 13, 15, 2, 0, "relu", 2), (1024, 128, 4, 4, 2, 2, "relu", 1)]


@pytest.mark.parametrize("cin,cout,h,w,batch,ksplit,act,stride", C3S_RES_CASES)
def test_small_map_3x3_kernel_residual(cin, cout, h, w, batch, ksplit, act, stride):
    from oracle import oracle as o
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    announce("small-map 3x3 + residual", cin, cout, h, w, batch, ksplit, act, stride)
    # layer 0 makes the input of the layer under test, layer 1 the residual operand (at the output's size)
    layers = [nets.conv(64, cin, 1, 1, 0, "relu"), nets.conv(cin, cout, 3, stride, 1, "relu"),
              nets.conv(cin, cout, 3, stride, 1, act, input_from=0, residual_from=1)]
    net = _mk(layers, h, w, 64, dist="normal")
    x, ws, bs = gen.make_params(net, batch, 15)
    B.dlf_debug_block3x3_mode(1, 5, ksplit, 0)
    try:
        s = Session(net, batch, ws, bs, **_manual(3, [0, 1, 2]))
    finally:
        B.dlf_debug_block3x3_mode(0)
    try:
        cfg = B.dlf_plan_group_config(s.plan, 2)
        assert cfg["kind"] == 10, cfg
        assert B.dlf_plan_group_io(s.plan, 2) == (0, 1)
        got = s.run_numpy(x)
    finally:
        s.close()
    compare(got, o.run_net(net, x, ws, bs), "small-map 3x3 + residual s%d %d->%d %dx%d" % (stride, cin, cout, h, w))


# (c, cout, height, width, batch, tile th, tile tw, act of the 3x3, act of the 1x1, residual): the fused
# 3x3 -> 1x1 kernel (shape 6 of the hook; th = 0: the planner's cut): two and four 32-pixel blocks per
# tile, ragged tiles at the map's edges, tiles of one row or one column, 128 and 256 channels, one and two slices of
# the second layer's channel blocks, a ragged last channel block, fewer channel blocks than waves, with
# and without the residual operand (which shares LDS with the region: 256 channels x 98 pixels go without)
C3PW_CASES = [(128, 512, 28, 28, 2, 7, 14, "relu", "relu", True), (128, 512, 28, 28, 1, 0, 0, "relu", "relu", True),
              (256, 1024, 14, 14, 2, 7, 7, "relu", "relu", True), (128, 512, 13, 17, 2, 8, 16, "relu6", "none", True),
              (128, 200, 9, 11, 3, 5, 6, "relu", "relu6", False), (256, 1024, 14, 14, 1, 7, 14, "relu", "relu", False),
              (128, 96, 5, 40, 1, 1, 16, "none", "relu", True), (256, 72, 19, 3, 2, 8, 1, "relu", "relu", False),
              (128, 1024, 7, 7, 2, 0, 0, "relu", "relu", True), (256, 520, 6, 6, 3, 3, 6, "relu", "relu", True),
              # 64 channels: workgroups of four waves, two to a CU; 256 and more output channels (two slices), a ragged block
              (64, 256, 56, 56, 1, 7, 14, "relu", "relu", True), (64, 256, 28, 28, 2, 0, 0, "relu", "relu", True),
              (64, 256, 13, 17, 2, 7, 8, "relu6", "none", True), (64, 520, 9, 11, 3, 5, 6, "relu", "relu", True),
              (64, 72, 5, 40, 1, 1, 16, "none", "relu", False), (64, 256, 19, 3, 2, 8, 1, "relu", "relu6", True)]


@pytest.mark.parametrize("c,cout,h,w,batch,th,tw,act1,act2,residual", C3PW_CASES)
def test_fused_3x3_pointwise_kernel(c, cout, h, w, batch, th, tw, act1, act2, residual):
    from oracle import oracle as o
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    announce("fused 3x3 -> 1x1", c, cout, h, w, batch, th, tw, act1, act2, residual)
    layers = [nets.conv(64, cout, 1, 1, 0, "relu"), nets.conv(cout, c, 1, 1, 0, "relu"), nets.conv(c, c, 3, 1, 1, act1),
              nets.conv(c, cout, 1, 1, 0, act2, **(dict(residual_from=0) if residual else {}))]
    net = _mk(layers, h, w, 64, dist="normal")
    x, ws, bs = gen.make_params(net, batch, 14)
    B.dlf_debug_block3x3_mode(1, 6, th, tw)        # shape 6: this kernel; th x tw: its tile
    try:
        s = Session(net, batch, ws, bs, **_manual(4, [0, 1, 3]))
    finally:
        B.dlf_debug_block3x3_mode(0)
    try:
        cfg = B.dlf_plan_group_config(s.plan, 2)
        assert cfg["kind"] == 11, cfg
        if th:      # the map is cut into equal tiles, as many as tiles of th x tw need
            gp = B.dlf_plan_groups(s.plan)[2]
            assert (gp["tile_h"], gp["tile_w"]) == (-(-h // -(-h // th)), -(-w // -(-w // tw))), gp
        got = s.run_numpy(x)
    finally:
        s.close()
    compare(got, o.run_net(net, x, ws, bs), "fused 3x3 -> 1x1 %d->%d %dx%d" % (c, cout, h, w))


# (cin0, cout, height, width, batch, tile th, tile tw, identity shortcut, activations of the three layers): a
# whole bottleneck block 1x1 -> 3x3 -> 1x1 on one kernel (shape 7 of the hook; th = 0: the planner's cut):
# tiles that divide the map and ragged ones, one-row and one-column tiles, 128 / 256 / 512 input
# channels, one and two slices of the last layer's channel blocks, a ragged last block, with the block's
# input as the residual operand and without
BNECK_CASES = [(256, 256, 56, 56, 1, 7, 8, True, ("relu", "relu", "relu")), (256, 256, 28, 28, 2, 0, 0, True, ("relu", "relu", "relu")),
               (128, 128, 13, 17, 2, 7, 8, True, ("relu6", "relu", "none")), (512, 512, 9, 11, 2, 5, 6, True, ("relu", "relu6", "relu")),
               (256, 520, 9, 11, 3, 4, 14, False, ("relu", "relu", "relu")), (128, 72, 5, 40, 1, 1, 16, False, ("none", "relu", "relu")),
               (256, 256, 19, 3, 2, 8, 1, True, ("relu", "none", "relu6")), (512, 200, 6, 6, 3, 3, 6, False, ("relu", "relu", "relu"))]


@pytest.mark.parametrize("cin0,cout,h,w,batch,th,tw,identity,acts", BNECK_CASES)
def test_bottleneck_kernel(cin0, cout, h, w, batch, th, tw, identity, acts):
    from oracle import oracle as o
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    announce("bottleneck", cin0, cout, h, w, batch, th, tw, identity, acts)
    layers = [nets.conv(32, cin0, 1, 1, 0, "relu"), nets.conv(cin0, 64, 1, 1, 0, acts[0]), nets.conv(64, 64, 3, 1, 1, acts[1]),
              nets.conv(64, cout, 1, 1, 0, acts[2], **(dict(residual_from=0) if identity else {}))]
    net = _mk(layers, h, w, 32, dist="normal")
    x, ws, bs = gen.make_params(net, batch, 16)
    B.dlf_debug_block3x3_mode(1, 7, th, tw)        # shape 7: this kernel; th x tw: its tile
    try:
        s = Session(net, batch, ws, bs, **_manual(4, [0, 3]))
    finally:
        B.dlf_debug_block3x3_mode(0)
    try:
        cfg = B.dlf_plan_group_config(s.plan, 1)
        assert cfg["kind"] == 12 and cfg["variant"] == cin0, cfg
        assert B.dlf_plan_group_io(s.plan, 1) == (0, -2)      # the shortcut is the group's own input
        if th:
            gp = B.dlf_plan_groups(s.plan)[1]
            assert (gp["tile_h"], gp["tile_w"]) == (-(-h // -(-h // th)), -(-w // -(-w // tw))), gp
        got = s.run_numpy(x)
    finally:
        s.close()
    compare(got, o.run_net(net, x, ws, bs), "bottleneck %d->64->64->%d %dx%d" % (cin0, cout, h, w))


# (cin0, height, width, batch, tile th, tile tw, activations): the same kernel without its last layer, the
# pair 1x1 -> 3x3 (64 channels out)
BNECK2_CASES = [(64, 56, 56, 1, 7, 8, ("relu", "relu")), (64, 28, 28, 2, 0, 0, ("relu", "relu")), (256, 13, 17, 2, 7, 8, ("relu6", "none")),
                (128, 9, 11, 3, 5, 6, ("none", "relu")), (512, 5, 40, 1, 1, 16, ("relu", "relu6")), (64, 19, 3, 2, 8, 1, ("relu", "relu"))]


@pytest.mark.parametrize("cin0,h,w,batch,th,tw,acts", BNECK2_CASES)
def test_bottleneck_kernel_two_layers(cin0, h, w, batch, th, tw, acts):
    from oracle import oracle as o
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    announce("bottleneck, two layers", cin0, h, w, batch, th, tw, acts)
    layers = [nets.conv(32, cin0, 1, 1, 0, "relu"), nets.conv(cin0, 64, 1, 1, 0, acts[0]), nets.conv(64, 64, 3, 1, 1, acts[1])]
    net = _mk(layers, h, w, 32, dist="normal")
    x, ws, bs = gen.make_params(net, batch, 17)
    B.dlf_debug_block3x3_mode(1, 7, th, tw)
    try:
        s = Session(net, batch, ws, bs, **_manual(3, [0, 2]))
    finally:
        B.dlf_debug_block3x3_mode(0)
    try:
        cfg = B.dlf_plan_group_config(s.plan, 1)
        assert cfg["kind"] == 12 and cfg["variant"] == cin0, cfg
        got = s.run_numpy(x)
    finally:
        s.close()
    compare(got, o.run_net(net, x, ws, bs), "1x1 -> 3x3 %d->64->64 %dx%d" % (cin0, h, w))


def test_pair_and_bottleneck_kernels_random_shapes():
    """Seeded random shapes for the 3x3 -> 1x1 pair kernel (64 / 128 / 256 channels) and the bottleneck
    kernel (two and three layers): maps that the tile does not divide, every tile size the hook lets
    through, odd output channel counts (multiples of 8), with and without the residual operand."""
    import random
    from oracle import oracle as o
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    rnd = random.Random(20252)
    done = 0
    tries = 0
    while done < 30 and tries < 400:
        tries += 1
        which = rnd.choice(("pair", "pair", "bneck3", "bneck2"))
        h, w = rnd.randint(1, 20), rnd.randint(1, 20)
        batch = rnd.randint(1, 3)
        th, tw = rnd.randint(1, 8), rnd.randint(1, 16)
        acts = [rnd.choice(("relu", "relu6", "none")) for _ in range(3)]
        residual = rnd.random() < 0.6
        if which == "pair":
            c = rnd.choice((64, 128, 256))
            cout = 8 * rnd.randint(1, 80)
            if th * tw > 128:
                continue
            layers = [nets.conv(16, cout, 1, 1, 0, "relu"), nets.conv(cout, c, 1, 1, 0, "relu"), nets.conv(c, c, 3, 1, 1, acts[0]),
                      nets.conv(c, cout, 1, 1, 0, acts[1], **(dict(residual_from=0) if residual else {}))]
            lasts, shape, kind, target = [0, 1, 3], 6, 11, 2
        elif which == "bneck3":
            cin0 = rnd.choice((128, 256, 512))
            cout = cin0 if residual else 8 * rnd.randint(1, 80)
            if th * tw > 64:
                continue
            layers = [nets.conv(16, cin0, 1, 1, 0, "relu"), nets.conv(cin0, 64, 1, 1, 0, acts[0]), nets.conv(64, 64, 3, 1, 1, acts[1]),
                      nets.conv(64, cout, 1, 1, 0, acts[2], **(dict(residual_from=0) if residual else {}))]
            lasts, shape, kind, target = [0, 3], 7, 12, 1
        else:
            cin0 = rnd.choice((64, 128, 256, 512))
            if th * tw > 64:
                continue
            layers = [nets.conv(16, cin0, 1, 1, 0, "relu"), nets.conv(cin0, 64, 1, 1, 0, acts[0]), nets.conv(64, 64, 3, 1, 1, acts[1])]
            lasts, shape, kind, target = [0, 2], 7, 12, 1
        net = _mk(layers, h, w, 16, dist="normal")
        x, ws, bs = gen.make_params(net, batch, 300 + done)
        B.dlf_debug_block3x3_mode(1, shape, th, tw)
        try:
            s = Session(net, batch, ws, bs, **_manual(len(layers), lasts, budget=rnd.choice((32, 256))))
        except B.DlfError:
            continue
        finally:
            B.dlf_debug_block3x3_mode(0)
        try:
            if B.dlf_plan_group_config(s.plan, target)["kind"] != kind:
                continue                  # the tile does not fit LDS: another kernel took the group
            announce("pair / bottleneck random", done, which, [L["cout"] for L in layers], h, w, batch, th, tw, acts, residual)
            got = s.run_numpy(x)
        finally:
            s.close()
        compare(got, o.run_net(net, x, ws, bs), "pair / bottleneck random case %d (%s)" % (done, which))
        done += 1
    assert done == 30


# (channels in, channels out, height, width, batch, activation): 1x1 layers on the same kernel (pointwise
# mode 8): chunks of 128 channels whole or split over the waves, 2 to 64 channel blocks, ragged last
# slices, tiles of fewer than 32 pixels, several tiles per map, a one-pixel map
C3S_PW_CASES = [(1024, 256, 14, 14, 2, "relu"), (512, 2048, 7, 7, 2, "relu"), (256, 64, 9, 11, 3, "none"),
                (1024, 1024, 7, 7, 1, "relu6"), (512, 200, 3, 5, 2, "relu"), (256, 1024, 1, 1, 4, "relu"),
                (1024, 96, 17, 8, 1, "relu"), (2048, 512, 7, 7, 2, "relu"), (2048, 72, 5, 3, 1, "none")]


@pytest.mark.parametrize("cin,cout,h,w,batch,act", C3S_PW_CASES)
def test_small_map_kernel_pointwise(cin, cout, h, w, batch, act):
    from oracle import oracle as o
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    announce("small-map 1x1", cin, cout, h, w, batch, act)
    net = _mk([nets.conv(cin, cout, 1, 1, 0, act)], h, w, cin, dist="normal")
    x, ws, bs = gen.make_params(net, batch, 13)
    B.dlf_debug_pointwise_mode(8)
    try:
        s = Session(net, batch, ws, bs, **_manual(1, [0]))
    finally:
        B.dlf_debug_pointwise_mode(0)
    try:
        cfg = B.dlf_plan_group_config(s.plan, 0)
        assert cfg["kind"] == 10 and cfg["variant"] >= 8, cfg
        got = s.run_numpy(x)
    finally:
        s.close()
    compare(got, o.run_net(net, x, ws, bs), "small-map 1x1 %d->%d %dx%d" % (cin, cout, h, w))


def test_block3x3_kernel_random_shapes():
    """Seeded random layers, block shapes, pixel tiles, budgets, batches, folded pools and residual
    operands for the block 3x3 kernel (every case one it accepts), against the oracle."""
    import random
    from oracle import oracle as o
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    rnd = random.Random(20240611)
    tile_h, tile_w = (2, 4, 7, 8, 14, 16), (4, 7, 8, 14, 16, 28, 32)
    wc, ach, fp = (2, 2, 1, 1, 2), (32, 64, 32, 64, 32), (2, 2, 2, 2, 4)
    done = tries = 0
    while done < 24 and tries < 2000:
        tries += 1
        shape = rnd.randrange(5)
        cin = rnd.choice((32, 64, 96, 128, 192))
        cout = rnd.choice((8, 24, 32, 40, 64, 72, 128, 136, 200))
        h, w = rnd.randint(3, 36), rnd.randint(3, 36)
        pool = rnd.random() < 0.3
        res = (not pool) and rnd.random() < 0.25
        th, tw = rnd.choice(tile_h), rnd.choice(tile_w)
        batch = rnd.randint(1, 3)
        act = rnd.choice(("relu", "relu6", "none"))
        if pool:
            h, w = h + (h & 1), w + (w & 1)
        if cin % ach[shape] or th * tw > 32 * fp[shape] * (8 // wc[shape]) or (pool and ((th | tw) & 1)):
            continue
        if cin * cout * h * w * batch > 2e8:
            continue
        if res:
            if cout % ach[shape]:
                continue
            layers = [nets.conv(cin, cout, 1, 1, 0, "relu"), nets.conv(cout, cout, 3, 1, 1, act, residual_from=0)]
            lasts = [0, 1]
        else:
            layers = [nets.conv(cin, cout, 3, 1, 1, act)]
            lasts = [0]
            if pool:
                layers.append(nets.maxpool(cout, 2, 2, 0))
                lasts = [1]
        net = _mk(layers, h, w, cin, dist="normal")
        x, ws, bs = gen.make_params(net, batch, 100 + done)
        B.dlf_debug_block3x3_mode(1, shape, th, tw)
        try:
            s = Session(net, batch, ws, bs, **_manual(len(layers), lasts, budget=rnd.choice((8, 64, 256))))
        except B.DlfError:
            continue                      # the shape does not fit LDS with this tile
        finally:
            B.dlf_debug_block3x3_mode(0)
        try:
            if B.dlf_plan_group_config(s.plan, len(lasts) - 1)["kind"] != 4:
                continue
            announce("block 3x3 random", done, cin, cout, h, w, batch, shape, th, tw, pool, res, act)
            got = s.run_numpy(x)
        finally:
            s.close()
        compare(got, o.run_net(net, x, ws, bs), "block 3x3 random case %d" % done)
        done += 1
    assert done == 24


@pytest.mark.parametrize("k_hw,k_c,cout,batch", [(8, 64, 1000, 3), (7, 96, 70, 40), (4, 512, 96, 16)])
def test_fc_split_k(k_hw, k_c, cout, batch):
    """Long K, few output channels: the planner splits K over workgroups (pairs of 32-channel
    blocks, an odd number of blocks and two batch blocks included) and a second launch adds the
    slices."""
    announce("fc split-K", k_hw, k_c, cout, batch)
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    layers = [nets.fc(k_hw * k_hw * k_c, cout, "relu")]
    net = _mk(layers, k_hw, k_hw, k_c, dist="normal")
    x, ws, bs = gen.make_params(net, batch)
    from oracle import oracle as o
    ref = o.run_net(net, x, ws, bs)
    for ksplit in (2, 4, 8):
        B.dlf_debug_force_config(1, 1, 0, ksplit, 0, 0, 32)
        try:
            s = Session(net, batch, ws, bs)
        finally:
            B.dlf_debug_force_config(0, 0, 0, 1, 0, 0, 32)
        try:
            assert B.dlf_plan_workspace_bytes(s.plan) > 0, "the split-K form keeps partial sums in the workspace"
            got = s.run_numpy(x)
        finally:
            s.close()
        compare(got, ref, "fc %d->%d batch %d, K in %d slices" % (k_hw * k_hw * k_c, cout, batch, ksplit))


# the last column: does the forced tile fit on-chip memory with a streaming first stage?  (a 16 x 16
# or 14 x 14 tile of 64 channels needs more than 8 vectors per data-movement thread and round)
@pytest.mark.parametrize("depth,c,hw,tile,streams", [(2, 16, 32, (8, 8), True), (3, 32, 21, (8, 8), True),
                                                     (4, 16, 19, (4, 8), True), (2, 64, 30, (16, 16), False),
                                                     (4, 64, 56, (14, 14), False)])
def test_fused_chain_equals_oracle(depth, c, hw, tile, streams):
    from paper_2011_05630_amd.binding import DlfError, DLF_ERR_INFEASIBLE
    announce("fused chain", depth, c, hw, tile)
    net = nets.identical_chain(c, hw, depth)
    for stream0 in (1, 0):
        for variant in (2, 0, 1):
            force = (tile[0], tile[1], variant, 1, 0, stream0)
            if stream0 and not streams:
                # the expected answer is an error status, not a crash and not a silent fallback
                with pytest.raises(DlfError) as e:
                    _run(net, 2, force=force, **_manual(depth, [depth - 1]))
                assert e.value.status == DLF_ERR_INFEASIBLE, e.value
                continue
            got, ref, g = _run(net, 2, force=force, **_manual(depth, [depth - 1]))
            assert len(g) == 1
            compare(got, ref, "chain d%d c%d stream%d v%d" % (depth, c, stream0, variant))


def test_fused_chain_with_strides_and_pool():
    announce("fused chain stride/pool")
    layers = [nets.conv(16, 32, 3, 2, 1, "relu"), nets.conv(32, 32, 3, 1, 1, "relu"),
              nets.maxpool(32, 3, 2, 1), nets.conv(32, 64, 1, 1, 0, "relu6")]
    net = _mk(layers, 45, 41, 16, dist="normal")
    got, ref, g = _run(net, 2, **_manual(4, [3]))
    assert len(g) == 1
    compare(got, ref, "conv s2 - conv - pool3x3s2 - conv1x1 fused")
    got, ref, g = _run(net, 2, **_manual(4, [0, 1, 2, 3]))
    compare(got, ref, "same, unfused")
