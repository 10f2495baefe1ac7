"""Pins for the numeric CPU oracle: each test ties one of its functions to something other than
itself (closed forms, hand values, library routines on special cases, invariants)."""
import numpy as np
import pytest
from scipy.signal import correlate2d

from oracle import oracle as o

RNG = np.random.default_rng(12345)
ACCS = ("f32", "f64")


def rnd(*shape):
    return RNG.standard_normal(shape).astype(np.float32)


@pytest.mark.parametrize("acc", ACCS)
def test_tap_count_closed_form(acc):
    # all-ones input and kernel, pad 1: each output counts the taps that land inside the image
    x = np.ones((1, 3, 3, 1), np.float32)
    w = np.ones((1, 3, 3, 1), np.float32)
    y = o.conv2d(x, w, None, 1, 1, acc=acc)[0, :, :, 0]
    assert np.array_equal(y, np.array([[4, 6, 4], [6, 9, 6], [4, 6, 4]], np.float32))
    # 5x4 image: (min(y+1,H-1)-max(y-1,0)+1) * (same in x)
    x = np.ones((2, 5, 4, 3), np.float32)
    w = np.ones((2, 3, 3, 3), np.float32)
    y = o.conv2d(x, w, None, 1, 1, acc=acc)
    for yy in range(5):
        for xx in range(4):
            ny = min(yy + 1, 4) - max(yy - 1, 0) + 1
            nx = min(xx + 1, 3) - max(xx - 1, 0) + 1
            assert np.all(y[:, yy, xx, :] == 3 * ny * nx)


@pytest.mark.parametrize("acc", ACCS)
def test_centre_delta_is_identity_plus_bias(acc):
    x = rnd(2, 6, 5, 4)
    w = np.zeros((4, 3, 3, 4), np.float32)
    for c in range(4):
        w[c, 1, 1, c] = 1.0
    b = np.array([0.5, -1.0, 0.0, 2.0], np.float32)
    y = o.conv2d(x, w, b, 1, 1, acc=acc)
    assert np.array_equal(y, x + b)


@pytest.mark.parametrize("kh,kw", [(0, 0), (0, 2), (2, 1), (1, 0), (2, 2)])
def test_off_centre_delta_shifts_with_zero_border(kh, kw):
    # w[co,kh,kw,ci] = delta(co,ci): out[y,x] = in[y-1+kh, x-1+kw], zero outside the image
    x = rnd(1, 5, 6, 3)
    w = np.zeros((3, 3, 3, 3), np.float32)
    for c in range(3):
        w[c, kh, kw, c] = 1.0
    y = o.conv2d(x, w, None, 1, 1)
    exp = np.zeros_like(x)
    for yy in range(5):
        for xx in range(6):
            iy, ix = yy - 1 + kh, xx - 1 + kw
            if 0 <= iy < 5 and 0 <= ix < 6:
                exp[0, yy, xx] = x[0, iy, ix]
    assert np.array_equal(y, exp)


def test_channel_index_order_of_weights():
    # w[co, kh, kw, ci]: a weight that picks input channel 2 into output channel 1 only
    x = rnd(1, 4, 4, 3)
    w = np.zeros((2, 1, 1, 3), np.float32)
    w[1, 0, 0, 2] = 2.0
    y = o.conv2d(x, w, None, 1, 0)
    assert np.array_equal(y[..., 0], np.zeros((1, 4, 4), np.float32))
    assert np.array_equal(y[..., 1], 2.0 * x[..., 2])


def test_linearity_at_zero_bias():
    x1, x2 = rnd(1, 7, 7, 5), rnd(1, 7, 7, 5)
    w = rnd(6, 3, 3, 5)
    a, b = np.float32(1.5), np.float32(-0.75)
    lhs = o.conv2d(a * x1 + b * x2, w, None, 1, 1, acc="f64")
    rhs = a * o.conv2d(x1, w, None, 1, 1, acc="f64") + b * o.conv2d(x2, w, None, 1, 1, acc="f64")
    assert np.allclose(lhs, rhs, rtol=1e-5, atol=1e-5)


@pytest.mark.parametrize("acc", ACCS)
def test_1x1_conv_is_matmul(acc):
    x = rnd(2, 5, 6, 7)
    w = rnd(9, 1, 1, 7)
    b = rnd(9)
    y = o.conv2d(x, w, b, 1, 0, acc=acc)
    ref = (x.reshape(-1, 7).astype(np.float64) @ w.reshape(9, 7).T.astype(np.float64)
           + b).reshape(2, 5, 6, 9)
    assert np.allclose(y, ref, rtol=1e-5, atol=1e-5)


@pytest.mark.parametrize("k,pad", [(3, 1), (5, 2), (7, 3)])
def test_single_channel_is_correlate2d(k, pad):
    x = rnd(1, 9, 8, 1)
    w = rnd(1, k, k, 1)
    y = o.conv2d(x, w, None, 1, pad, acc="f64")[0, :, :, 0]
    ref = correlate2d(x[0, :, :, 0].astype(np.float64), w[0, :, :, 0].astype(np.float64),
                      mode="same")
    assert np.allclose(y, ref, rtol=1e-5, atol=1e-5)


def test_multichannel_is_sum_of_correlations():
    x = rnd(1, 6, 7, 3)
    w = rnd(2, 3, 3, 3)
    y = o.conv2d(x, w, None, 1, 1, acc="f64")
    for co in range(2):
        ref = sum(correlate2d(x[0, :, :, ci].astype(np.float64), w[co, :, :, ci].astype(np.float64),
                              mode="same") for ci in range(3))
        assert np.allclose(y[0, :, :, co], ref, rtol=1e-5, atol=1e-5)


@pytest.mark.parametrize("h,w_", [(8, 8), (7, 9), (5, 5)])
def test_stride2_is_subsampled_stride1(h, w_):
    x = rnd(2, h, w_, 3)
    w = rnd(4, 3, 3, 3)
    b = rnd(4)
    y1 = o.conv2d(x, w, b, 1, 1)
    y2 = o.conv2d(x, w, b, 2, 1)
    assert y2.shape == (2, (h + 2 - 3) // 2 + 1, (w_ + 2 - 3) // 2 + 1, 4)
    assert np.array_equal(y2, y1[:, ::2, ::2, :])


@pytest.mark.parametrize("k,stride,pad,groups", [(3, 1, 1, 1), (3, 2, 1, 1), (1, 1, 0, 1), (1, 2, 0, 1),
                                                 (7, 2, 3, 1), (5, 1, 2, 1), (3, 1, 1, 6), (3, 2, 1, 6),
                                                 (11, 4, 2, 1)])
def test_conv2d_agrees_with_torch_cpu_as_a_third_opinion(k, stride, pad, groups):
    """torch.nn.functional.conv2d on the CPU (NCHW, its own kernels) on random tensors: every
    filter size, stride and padding the workloads use, dense and depthwise (groups = channels)."""
    import torch
    import torch.nn.functional as F
    cin, cout = 6, 6 if groups > 1 else 5
    x = rnd(2, 13, 17, cin)
    w = rnd(cout, k, k, cin // groups)
    b = rnd(cout)
    want = F.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2).double(),
                    torch.from_numpy(w).permute(0, 3, 1, 2).double(), torch.from_numpy(b).double(),
                    stride=stride, padding=pad, groups=groups).permute(0, 2, 3, 1).numpy()
    for acc, tol in (("f32", 2e-5), ("f64", 2e-6)):
        got = o.conv2d(x, w, b, stride, pad, groups=groups, acc=acc)
        assert got.shape == want.shape
        assert np.abs(got - want).max() <= tol * max(1.0, np.abs(want).max())


def test_maxpool_and_fc_agree_with_torch_cpu():
    import torch
    import torch.nn.functional as F
    x = rnd(2, 9, 11, 4)
    for k, s, p in ((2, 2, 0), (3, 2, 1), (3, 2, 0)):
        want = F.max_pool2d(torch.from_numpy(x).permute(0, 3, 1, 2), k, s, p).permute(0, 2, 3, 1).numpy()
        assert np.array_equal(o.maxpool(x, k, s, p), want)
    xf = rnd(3, 40)
    w = rnd(7, 40)
    b = rnd(7)
    want = F.linear(torch.from_numpy(xf).double(), torch.from_numpy(w).double(), torch.from_numpy(b).double()).numpy()
    assert np.abs(o.fc(xf, w, b, acc="f64") - want).max() <= 1e-5


def test_stride2_5x5_hand_case():
    # 5x5 ramp, 3x3 box kernel, stride 2, pad 1 -> 3x3 window sums, by hand
    x = np.arange(25, dtype=np.float32).reshape(1, 5, 5, 1)
    w = np.ones((1, 3, 3, 1), np.float32)
    y = o.conv2d(x, w, None, 2, 1)[0, :, :, 0]
    exp = np.array([[0 + 1 + 5 + 6, 1 + 2 + 3 + 6 + 7 + 8, 3 + 4 + 8 + 9],
                    [5 + 6 + 10 + 11 + 15 + 16, 6 + 7 + 8 + 11 + 12 + 13 + 16 + 17 + 18,
                     8 + 9 + 13 + 14 + 18 + 19],
                    [15 + 16 + 20 + 21, 16 + 17 + 18 + 21 + 22 + 23, 18 + 19 + 23 + 24]],
                   np.float32)
    assert np.array_equal(y, exp)


def test_7x7_stride2_pad3_output_size_and_corner():
    x = np.ones((1, 10, 10, 2), np.float32)
    w = np.ones((1, 7, 7, 2), np.float32)
    y = o.conv2d(x, w, None, 2, 3)
    assert y.shape == (1, 5, 5, 1)
    assert y[0, 0, 0, 0] == 4 * 4 * 2        # rows/cols 0..3 inside
    assert y[0, 2, 2, 0] == 7 * 7 * 2        # centre 4: rows 1..7 inside


@pytest.mark.parametrize("stride", [1, 2])
def test_depthwise_is_per_channel_correlation(stride):
    x = rnd(2, 7, 6, 5)
    w = rnd(5, 3, 3, 1)
    b = rnd(5)
    y = o.conv2d(x, w, b, stride, 1, groups=5, acc="f64")
    for n in range(2):
        for c in range(5):
            ref = correlate2d(x[n, :, :, c].astype(np.float64), w[c, :, :, 0].astype(np.float64),
                              mode="same")[::stride, ::stride] + b[c]
            assert np.allclose(y[n, :, :, c], ref, rtol=1e-5, atol=1e-5)


def test_grouped_conv_matches_per_group_dense():
    x = rnd(1, 5, 5, 6)
    w = rnd(4, 3, 3, 3)   # 2 groups: 3 in, 2 out each
    y = o.conv2d(x, w, None, 1, 1, groups=2)
    y0 = o.conv2d(x[..., :3], w[:2], None, 1, 1)
    y1 = o.conv2d(x[..., 3:], w[2:], None, 1, 1)
    assert np.array_equal(y, np.concatenate([y0, y1], axis=-1))


@pytest.mark.parametrize("acc", ACCS)
def test_fc_is_matmul_and_uses_nhwc_flatten(acc):
    x = rnd(3, 2, 2, 5)
    w = rnd(7, 20)
    b = rnd(7)
    y = o.fc(x.reshape(3, -1), w, b, acc=acc)
    ref = x.reshape(3, 20).astype(np.float64) @ w.T.astype(np.float64) + b
    assert np.allclose(y, ref, rtol=1e-5, atol=1e-5)
    # apply_layer flattens in (h, w, c) order
    L = dict(op="fc", cin=20, cout=7, kh=1, kw=1, stride=1, pad=0, has_bias=1, act="none",
             input_from=-1, residual_from=-1)
    y2 = o.apply_layer(L, x, w.reshape(7, 1, 1, 20), b, acc=acc)
    assert np.array_equal(y2.reshape(3, 7), y)


def test_f32_accumulation_order_is_kh_kw_ci():
    # fp32 sum in the documented order, replayed in numpy with explicit float32 adds
    x = rnd(1, 3, 3, 4)
    w = rnd(1, 3, 3, 4)
    b = np.array([0.25], np.float32)
    y = o.conv2d(x, w, b, 1, 1)[0, 1, 1, 0]
    acc = np.float32(0.25)
    for kh in range(3):
        for kw in range(3):
            for ci in range(4):
                acc = np.float32(acc + np.float32(x[0, kh, kw, ci] * w[0, kh, kw, ci]))
    assert y == acc


def test_activations_hand_values():
    x = np.array([-2.0, -0.0, 0.0, 0.5, 6.0, 6.5, 100.0], np.float32)
    assert np.array_equal(o.act(x, "relu"), np.array([0, 0, 0, 0.5, 6.0, 6.5, 100.0], np.float32))
    assert np.array_equal(o.act(x, "relu6"), np.array([0, 0, 0, 0.5, 6.0, 6.0, 6.0], np.float32))
    assert np.array_equal(o.act(x, "none"), x)


def test_maxpool_2x2_is_reshape_max_and_handles_ties_and_negatives():
    x = rnd(2, 6, 8, 3)
    x[0, 0, 0, 0] = x[0, 0, 1, 0] = 5.0      # tie
    x[1, 2:4, 2:4, 1] = -3.0                 # all-negative window
    y = o.maxpool(x, 2, 2, 0)
    ref = x.reshape(2, 3, 2, 4, 2, 3).max(axis=(2, 4))
    assert np.array_equal(y, ref)
    assert y[1, 1, 1, 1] == -3.0


def test_maxpool_3x3_s2_p1_pads_with_minus_infinity():
    x = -np.ones((1, 4, 4, 1), np.float32) * np.arange(1, 17, dtype=np.float32).reshape(1, 4, 4, 1)
    y = o.maxpool(x, 3, 2, 1)[0, :, :, 0]
    # all inputs negative: a zero pad would win everywhere; -inf padding must not
    exp = np.array([[-1, -2], [-5, -6]], np.float32)
    assert np.array_equal(y, exp)


@pytest.mark.parametrize("acc", ACCS)
def test_global_avgpool_is_mean(acc):
    x = rnd(2, 7, 7, 5)
    y = o.global_avgpool(x, acc=acc)
    assert y.shape == (2, 1, 1, 5)
    assert np.allclose(y[:, 0, 0, :], x.astype(np.float64).mean(axis=(1, 2)), rtol=1e-5, atol=1e-6)


def test_residual_add_then_relu_hand_values():
    L = dict(op="conv", cin=1, cout=1, kh=1, kw=1, stride=1, pad=0, has_bias=1, act="relu",
             input_from=-1, residual_from=0)
    x = np.array([1.0, -2.0, 3.0, -4.0], np.float32).reshape(1, 2, 2, 1)
    skip = np.array([-3.0, 1.0, 1.0, 5.0], np.float32).reshape(1, 2, 2, 1)
    w = np.array([2.0], np.float32).reshape(1, 1, 1, 1)
    b = np.array([0.5], np.float32)
    y = o.apply_layer(L, x, w, b, residual=skip)
    # relu(2x + 0.5 + skip) = relu([-0.5, -2.5, 7.5, -2.5])
    assert np.array_equal(y.ravel(), np.array([0.0, 0.0, 7.5, 0.0], np.float32))


def test_run_net_projection_bottleneck_equals_manual_composition():
    from synth import nets
    layers = []
    layers.append(nets.conv(4, 4, 3, 1, 1, "relu"))              # 0: produces block input
    nets._bottleneck(layers, 4, 2, 2, True)                     # 1..4
    net = dict(layers=layers, in_h=6, in_w=6, in_c=4)
    x = rnd(1, 6, 6, 4)
    ws = [rnd(L["cout"], L["kh"], L["kw"], L["cin"]) for L in layers]
    bs = [rnd(L["cout"]) for L in layers]
    y = o.run_net(net, x, ws, bs)
    t0 = o.act(o.conv2d(x, ws[0], bs[0], 1, 1), "relu")
    a = o.act(o.conv2d(t0, ws[1], bs[1], 1, 0), "relu")
    b3 = o.act(o.conv2d(a, ws[2], bs[2], 2, 1), "relu")
    proj = o.conv2d(t0, ws[3], bs[3], 2, 0)
    out = o.act(o.conv2d(b3, ws[4], bs[4], 1, 0) + proj, "relu")
    assert np.array_equal(y, out)


def test_run_net_subrange_with_given_tensors():
    from synth import nets
    net = dict(layers=nets.conv_chain(3, 3), in_h=5, in_w=5, in_c=3)
    x = rnd(1, 5, 5, 3)
    ws = [rnd(3, 3, 3, 3) for _ in range(3)]
    bs = [rnd(3) for _ in range(3)]
    allo = o.run_net(net, x, ws, bs, keep_all=True)
    part = o.run_net(net, None, ws, bs, first=1, last=2, given={0: allo[0], -1: x})
    assert np.array_equal(part, allo[2])


def _chain(depth, c, stride_last=1):
    from synth import nets
    layers = nets.conv_chain(c, depth)
    if stride_last != 1:
        layers[-1] = nets.conv(c, c, 3, stride_last, 1, "relu")
    return layers


@pytest.mark.parametrize("depth", [2, 3])
def test_fused_tile_equals_unfused_bitwise_every_origin(depth):
    # brute force over every tile origin of a 6x6x2 image, including all borders
    layers = _chain(depth, 2)
    x = rnd(1, 6, 6, 2)
    ws = [rnd(2, 3, 3, 2) for _ in layers]
    bs = [rnd(2) + 0.3 for _ in layers]
    net = dict(layers=layers, in_h=6, in_w=6, in_c=2)
    full = o.run_net(net, x, ws, bs)
    for th, tw in [(2, 2), (3, 2), (6, 6)]:
        for oy in range(0, 6 - th + 1):
            for ox in range(0, 6 - tw + 1):
                t = o.fused_conv_tile(layers, x, ws, bs, oy, ox, th, tw, masked=True)
                assert np.array_equal(t, full[:, oy:oy + th, ox:ox + tw, :]), (oy, ox, th, tw)


def test_fused_tile_without_masking_differs_at_borders_only():
    layers = _chain(2, 2)
    x = rnd(1, 6, 6, 2)
    ws = [rnd(2, 3, 3, 2) for _ in layers]
    bs = [np.abs(rnd(2)) + 0.5 for _ in layers]      # positive bias: relu(bias) != 0 outside
    net = dict(layers=layers, in_h=6, in_w=6, in_c=2)
    full = o.run_net(net, x, ws, bs)
    border = o.fused_conv_tile(layers, x, ws, bs, 0, 0, 2, 2, masked=False)
    assert not np.array_equal(border, full[:, 0:2, 0:2, :])
    inner = o.fused_conv_tile(layers, x, ws, bs, 2, 2, 2, 2, masked=False)
    assert np.array_equal(inner, full[:, 2:4, 2:4, :])


def test_fused_tile_with_stride2_last_layer():
    layers = _chain(2, 2, stride_last=2)
    x = rnd(2, 7, 7, 2)
    ws = [rnd(2, 3, 3, 2) for _ in layers]
    bs = [rnd(2) for _ in layers]
    net = dict(layers=layers, in_h=7, in_w=7, in_c=2)
    full = o.run_net(net, x, ws, bs)
    assert full.shape == (2, 4, 4, 2)
    for oy in range(0, 3):
        for ox in range(0, 3):
            t = o.fused_conv_tile(layers, x, ws, bs, oy, ox, 2, 2)
            assert np.array_equal(t, full[:, oy:oy + 2, ox:ox + 2, :])


def test_round_intermediates_only_changes_by_fp16_rounding():
    from synth import nets, gen
    net = nets.two_layer_block()
    x, ws, bs = gen.make_params(net, 1)
    y32 = o.run_net(net, x, ws, bs)
    y16 = o.run_net(net, x, ws, bs, round_intermediates=True)
    rel = np.linalg.norm(y16 - y32) / np.linalg.norm(y32)
    assert 0 < rel < 2e-3


def test_f32_and_f64_accumulators_agree_on_config1():
    from synth import nets, gen
    net = nets.two_layer_block()
    x, ws, bs = gen.make_params(net, 1)
    y32 = o.run_net(net, x, ws, bs, acc="f32")
    y64 = o.run_net(net, x, ws, bs, acc="f64")
    assert np.allclose(y32, y64, rtol=1e-5, atol=1e-5)
    assert y32.shape == (1, 32, 32, 16)
