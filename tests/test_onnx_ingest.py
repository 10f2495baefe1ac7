"""The ONNX front end (the model-ingest step of the tool chain, Sec. IV-C): wire-format decoder
against hand-assembled bytes of the published protobuf encoding, round trips of the synthetic
networks through ONNX files, and the layout conversions (weights OIHW -> OHWI, the (c, h, w)
flattening in front of a fully connected layer, batch-norm folding) against an NCHW computation
with torch's CPU operators, evaluated through the oracle.  No ONNX package is installed here: files
come from tests/onnx_writer.py, so agreement with files of other exporters is "parity unpinned"."""
import numpy as np
import pytest

from paper_2011_05630_amd import onnx_ingest as oi
from synth import gen, nets
from tests import onnx_writer as ow


def test_wire_format_hand_bytes():
    # the encoding's own worked example: field 1, varint 150 -> 08 96 01
    assert list(oi._fields(bytes([0x08, 0x96, 0x01]))) == [(1, 0, 150)]
    # field 2, length-delimited "testing" -> 12 07 74 65 73 74 69 6e 67
    (f, wt, v), = list(oi._fields(bytes([0x12, 0x07]) + b"testing"))
    assert (f, wt, bytes(v)) == (2, 2, b"testing")
    # 300 -> AC 02; -1 as a 64-bit two's-complement varint: nine FF bytes and 01
    assert oi._varint(bytes([0xAC, 0x02]), 0) == (300, 2)
    v, pos = oi._varint(bytes([0xFF] * 9 + [0x01]), 0)
    assert (oi._signed64(v), pos) == (-1, 10)
    # packed repeated varints 3, 270, 86942 -> 03 8E 02 9E A7 05
    assert oi._packed_varints(memoryview(bytes([0x03, 0x8E, 0x02, 0x9E, 0xA7, 0x05])), 2) == [3, 270, 86942]
    # a 32-bit field holding the float 1.0 (00 00 80 3F) under field 2
    assert list(oi._fields(bytes([0x15, 0x00, 0x00, 0x80, 0x3F]))) == [(2, 5, 0x3F800000)]
    with pytest.raises(oi.OnnxIngestError):
        list(oi._fields(bytes([0x12, 0x07, 0x74])))          # length runs past the end


def test_tensor_encodings():
    a = np.arange(6, dtype=np.float32).reshape(2, 3) - 2.5
    name, got = oi._parse_tensor(ow.tensor("x", a))
    assert name == "x" and got.dtype == np.float32 and np.array_equal(got, a)
    # the same values as repeated float_data (field 4, packed) instead of raw bytes
    body = ow.f_varint(1, 2) + ow.f_varint(1, 3) + ow.f_varint(2, 1) + ow.f_bytes(4, a.tobytes())
    assert np.array_equal(oi._parse_tensor(body)[1], a)
    # fp16 as bit patterns in int32_data
    h = np.array([1.0, -2.0, 0.5], np.float16)
    body = ow.f_varint(1, 3) + ow.f_varint(2, 10) + ow.f_bytes(5, b"".join(ow.varint(int(b)) for b in h.view(np.uint16)))
    assert np.array_equal(oi._parse_tensor(body)[1], h)
    i64 = np.array([-1, 7], np.int64)
    assert np.array_equal(oi._parse_tensor(ow.tensor("s", i64))[1], i64)


def _same_net(a, b):
    assert (a["in_h"], a["in_w"], a["in_c"]) == (b["in_h"], b["in_w"], b["in_c"])
    assert len(a["layers"]) == len(b["layers"])
    for i, (la, lb) in enumerate(zip(a["layers"], b["layers"])):
        assert la == lb, (i, la, lb)


@pytest.mark.parametrize("make", [nets.two_layer_block, lambda: nets.vgg16(in_hw=32),
                                  lambda: nets.resnet50(in_hw=64), lambda: nets.resnet18(in_hw=64),
                                  lambda: nets.mobilenet_v1(in_hw=32), lambda: nets.alexnet(in_hw=224)])
@pytest.mark.parametrize("style", [dict(), dict(clip_as_inputs=False, packed=False)])
def test_round_trip_of_the_synthetic_networks(make, style):
    net = make()
    x, ws, bs = gen.make_params(net, 1)
    got_net, got_w, got_b = oi.load_onnx(ow.net_to_onnx(net, ws, bs, **style))
    _same_net(got_net, net)
    for i, (w, b) in enumerate(zip(ws, bs)):
        if w is None:
            assert got_w[i] is None and got_b[i] is None
        else:
            assert got_w[i].dtype == np.float16 and got_w[i].shape == w.shape and np.array_equal(got_w[i], w), i
            assert got_b[i].dtype == np.float32 and np.array_equal(got_b[i], b), i


def _fp16_exact(rng, shape, scale):
    return (rng.standard_normal(shape) * scale).astype(np.float16).astype(np.float32)


def test_layouts_and_batchnorm_folding_against_an_nchw_computation():
    """conv + BN + relu, maxpool, depthwise conv + relu6, 1x1 conv + residual add + relu, flatten,
    Gemm: torch computes it NCHW from the ONNX-layout tensors; the ingested layer list runs through
    the oracle NHWC."""
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    from oracle import oracle as o
    rng = np.random.default_rng(5)
    C0, C1, H = 3, 8, 12
    w0 = _fp16_exact(rng, (C1, C0, 3, 3), 0.3); b0 = rng.uniform(-0.1, 0.1, C1).astype(np.float32)
    bn = [rng.uniform(0.5, 1.5, C1).astype(np.float32), rng.uniform(-0.2, 0.2, C1).astype(np.float32),
          rng.uniform(-0.3, 0.3, C1).astype(np.float32), rng.uniform(0.5, 2.0, C1).astype(np.float32)]
    wd = _fp16_exact(rng, (C1, 1, 3, 3), 0.4); bd = rng.uniform(-0.1, 0.1, C1).astype(np.float32)
    wp = _fp16_exact(rng, (C1, C1, 1, 1), 0.3); bp = rng.uniform(-0.1, 0.1, C1).astype(np.float32)
    Hp = H // 2
    wf = _fp16_exact(rng, (10, C1 * Hp * Hp), 0.1); bf = rng.uniform(-0.1, 0.1, 10).astype(np.float32)
    nodes = [
        ow.node("Conv", ["input", "w0", "b0"], ["c0"], [ow.attr_ints("kernel_shape", [3, 3]), ow.attr_ints("pads", [1, 1, 1, 1])]),
        ow.node("BatchNormalization", ["c0", "g", "beta", "mu", "var"], ["n0"], [ow.attr_float("epsilon", 1e-3)]),
        ow.node("Relu", ["n0"], ["r0"]),
        ow.node("MaxPool", ["r0"], ["p0"], [ow.attr_ints("kernel_shape", [2, 2]), ow.attr_ints("strides", [2, 2])]),
        ow.node("Conv", ["p0", "wd", "bd"], ["d0"], [ow.attr_ints("kernel_shape", [3, 3]), ow.attr_ints("pads", [1, 1, 1, 1]), ow.attr_int("group", C1)]),
        ow.node("Clip", ["d0", "lo", "hi"], ["d0a"]),
        ow.node("Conv", ["d0a", "wp", "bp"], ["q0"], [ow.attr_ints("kernel_shape", [1, 1])]),
        ow.node("Add", ["d0a", "q0"], ["s0"]),            # skip operand first, branch end second
        ow.node("Relu", ["s0"], ["s0a"]),
        ow.node("Flatten", ["s0a"], ["fl"], [ow.attr_int("axis", 1)]),
        ow.node("Gemm", ["fl", "wf", "bf"], ["out"], [ow.attr_int("transB", 1)]),
    ]
    inits = [ow.tensor(n, a) for n, a in [("w0", w0), ("b0", b0), ("g", bn[0]), ("beta", bn[1]), ("mu", bn[2]),
                                           ("var", bn[3]), ("wd", wd), ("bd", bd), ("wp", wp), ("bp", bp),
                                           ("wf", wf), ("bf", bf), ("lo", np.array(0, np.float32)),
                                           ("hi", np.array(6, np.float32))]]
    data = ow.model(nodes, inits, [ow.value_info("input", [2, C0, H, H])], [ow.value_info("out", [2, 10])])
    net, ws, bs = oi.load_onnx(data)
    assert [L["op"] for L in net["layers"]] == ["conv", "maxpool", "dwconv", "conv", "fc"]
    assert [L["act"] for L in net["layers"]] == ["relu", "none", "relu6", "relu", "none"]
    assert net["layers"][3]["residual_from"] == 2 and (net["in_h"], net["in_w"], net["in_c"]) == (H, H, C0)

    x = rng.standard_normal((2, C0, H, H)).astype(np.float16).astype(np.float32)
    t = torch.from_numpy
    y = F.conv2d(t(x).double(), t(w0).double(), t(b0).double(), padding=1)
    y = F.batch_norm(y, t(bn[2]).double(), t(bn[3]).double(), t(bn[0]).double(), t(bn[1]).double(), False, 0.0, 1e-3)
    y = F.max_pool2d(F.relu(y), 2)
    d = torch.clamp(F.conv2d(y, t(wd).double(), t(bd).double(), padding=1, groups=C1), 0.0, 6.0)
    s = F.relu(F.conv2d(d, t(wp).double(), t(bp).double()) + d)
    ref = F.linear(s.flatten(1), t(wf).double(), t(bf).double()).numpy()

    got = o.run_net(net, np.ascontiguousarray(x.transpose(0, 2, 3, 1)), ws, bs, acc="f64")
    got = np.asarray(got).reshape(2, 10)
    # the folded weights are rounded to fp16 once more: that rounding bounds the difference
    assert np.abs(got - ref).max() <= 2e-2 * np.abs(ref).max(), (np.abs(got - ref).max(), np.abs(ref).max())
    # with the batch norm an identity (scale 1, shift 0, mean 0, var 1 - eps) nothing is re-rounded
    ident = [np.ones(C1, np.float32), np.zeros(C1, np.float32), np.zeros(C1, np.float32), np.full(C1, 1 - 1e-3, np.float32)]
    inits2 = [ow.tensor(n, a) for n, a in [("g", ident[0]), ("beta", ident[1]), ("mu", ident[2]), ("var", ident[3])]]
    keep = [i for i in inits if not any(i == ow.tensor(n, a) for n, a in [("g", bn[0]), ("beta", bn[1]), ("mu", bn[2]), ("var", bn[3])])]
    net2, ws2, bs2 = oi.load_onnx(ow.model(nodes, keep + inits2, [ow.value_info("input", [2, C0, H, H])],
                                           [ow.value_info("out", [2, 10])]))
    y = F.conv2d(t(x).double(), t(w0).double(), t(b0).double(), padding=1)
    y = F.max_pool2d(F.relu(y), 2)
    d = torch.clamp(F.conv2d(y, t(wd).double(), t(bd).double(), padding=1, groups=C1), 0.0, 6.0)
    s = F.relu(F.conv2d(d, t(wp).double(), t(bp).double()) + d)
    ref2 = F.linear(s.flatten(1), t(wf).double(), t(bf).double()).numpy()
    got2 = np.asarray(o.run_net(net2, np.ascontiguousarray(x.transpose(0, 2, 3, 1)), ws2, bs2, acc="f64")).reshape(2, 10)
    assert np.abs(got2 - ref2).max() <= 1e-5 * np.abs(ref2).max()


@pytest.mark.parametrize("bad", ["op", "dilation", "clip", "pads", "input"])
def test_unsupported_graphs_are_rejected(bad):
    w = np.zeros((4, 4, 3, 3), np.float32)
    attrs = [ow.attr_ints("kernel_shape", [3, 3]), ow.attr_ints("pads", [1, 1, 1, 1] if bad != "pads" else [1, 0, 1, 0])]
    if bad == "dilation":
        attrs.append(ow.attr_ints("dilations", [2, 2]))
    nodes = [ow.node("Conv", ["input", "w"], ["c"], attrs)]
    inits = [ow.tensor("w", w)]
    out = "c"
    if bad == "op":
        nodes.append(ow.node("Sigmoid", ["c"], ["s"]))
        out = "s"
    if bad == "clip":
        nodes.append(ow.node("Clip", ["c"], ["s"], [ow.attr_float("min", 0.0), ow.attr_float("max", 4.0)]))
        out = "s"
    shape = [1, 4, 8, 8] if bad != "input" else [1, 4]
    data = ow.model(nodes, inits, [ow.value_info("input", shape)], [ow.value_info(out, [1, 4, 8, 8])])
    with pytest.raises(oi.OnnxIngestError):
        oi.load_onnx(data)


@pytest.mark.gpu
@pytest.mark.parametrize("make,batch", [(lambda: nets.mobilenet_v1(in_hw=64), 3), (lambda: nets.resnet50(in_hw=64), 2)])
def test_ingested_network_runs_on_the_gpu(make, batch):
    """ONNX bytes -> layer list -> dlf_net_create / dlf_plan / dlf_run, against the oracle on the
    network the file was written from."""
    from oracle import oracle as o
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    from tests.gpu_util import announce, compare
    net = make()
    x, ws, bs = gen.make_params(net, batch)
    announce("onnx ingest", net["name"], "batch", batch)
    inet, iw, ib = oi.load_onnx(ow.net_to_onnx(net, ws, bs, batch=batch))
    s = Session(inet, batch, iw, ib, mode=B.TUNER_DP)
    got = s.run_numpy(x)
    s.close()
    compare(got, o.run_net(net, x, ws, bs), "onnx %s b=%d" % (net["name"], batch))
