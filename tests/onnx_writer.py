"""Writes ONNX model files for the ingest tests: an encoder of the protobuf wire format plus the
ONNX messages a CNN needs (test infrastructure; the product only reads ONNX).  Tensors are stored
as fp32 raw data, activations are declared NCHW, convolution weights are [Cout][Cin/group][kh][kw]
and a fully connected layer behind a feature map has its columns in (c, h, w) order, as an exporter
of an NCHW framework would write them."""
import struct

import numpy as np

from synth import nets


def varint(v):
    if v < 0:
        v += 1 << 64
    out = bytearray()
    while True:
        b = v & 0x7F
        v >>= 7
        if v:
            out.append(b | 0x80)
        else:
            out.append(b)
            return bytes(out)


def key(field, wt):
    return varint((field << 3) | wt)


def f_varint(field, v):
    return key(field, 0) + varint(int(v))


def f_bytes(field, b):
    if isinstance(b, str):
        b = b.encode("utf-8")
    return key(field, 2) + varint(len(b)) + bytes(b)


def f_float(field, v):
    return key(field, 5) + struct.pack("<f", v)


def tensor(name, arr):
    arr = np.ascontiguousarray(arr)
    dtype = {np.dtype("float32"): 1, np.dtype("int64"): 7, np.dtype("float16"): 10}[arr.dtype]
    out = b"".join(f_varint(1, d) for d in arr.shape)
    out += f_varint(2, dtype) + f_bytes(8, name) + f_bytes(9, arr.tobytes())
    return out


def attr_ints(name, vals, packed=True):
    body = f_bytes(1, name)
    if packed:
        body += f_bytes(8, b"".join(varint(v) for v in vals))
    else:
        body += b"".join(f_varint(8, v) for v in vals)
    return body + f_varint(20, 7)


def attr_int(name, v):
    return f_bytes(1, name) + f_varint(3, v) + f_varint(20, 2)


def attr_float(name, v):
    return f_bytes(1, name) + f_float(2, v) + f_varint(20, 1)


def node(op, inputs, outputs, attrs=(), name=""):
    out = b"".join(f_bytes(1, i) for i in inputs) + b"".join(f_bytes(2, o) for o in outputs)
    out += f_bytes(3, name or outputs[0]) + f_bytes(4, op)
    out += b"".join(f_bytes(5, a) for a in attrs)
    return out


def value_info(name, shape):
    dims = b"".join(f_bytes(1, f_varint(1, d)) for d in shape)
    ttype = f_varint(1, 1) + f_bytes(2, dims)
    return f_bytes(1, name) + f_bytes(2, f_bytes(1, ttype))


def model(nodes, initializers, inputs, outputs, opset=13):
    g = b"".join(f_bytes(1, n) for n in nodes) + f_bytes(2, "g")
    g += b"".join(f_bytes(5, t) for t in initializers)
    g += b"".join(f_bytes(11, v) for v in inputs) + b"".join(f_bytes(12, v) for v in outputs)
    return f_varint(1, 8) + f_bytes(2, "tests") + f_bytes(7, g) + f_bytes(8, f_bytes(1, "") + f_varint(2, opset))


def net_to_onnx(net, weights, biases, batch=1, clip_as_inputs=True, packed=True):
    """The layer list of synth.nets as an ONNX graph (opset 13 by default; clip_as_inputs=False
    writes ReLU6 as an opset-6 Clip with min / max attributes)."""
    shapes = nets.infer_shapes(net)
    nodes, inits = [], []
    out_name = {}                                    # layer index -> name of its final tensor
    cur = "input"
    flat = False
    if clip_as_inputs:
        inits += [tensor("clip_lo", np.array(0.0, np.float32)), tensor("clip_hi", np.array(6.0, np.float32))]
    for i, L in enumerate(net["layers"]):
        (h, w, c), (oh, ow, oc) = shapes[i]
        x = cur if L["input_from"] < 0 else out_name[L["input_from"]]
        t = "t%d" % i
        if L["op"] in ("conv", "dwconv"):
            W = weights[i].astype(np.float32).transpose(0, 3, 1, 2)          # OHWI -> OIHW
            inits += [tensor("w%d" % i, W), tensor("b%d" % i, biases[i].astype(np.float32))]
            attrs = [attr_ints("kernel_shape", [L["kh"], L["kw"]], packed),
                     attr_ints("strides", [L["stride"]] * 2, packed),
                     attr_ints("pads", [L["pad"]] * 4, packed),
                     attr_int("group", c if L["op"] == "dwconv" else 1)]
            nodes.append(node("Conv", [x, "w%d" % i, "b%d" % i], [t], attrs))
        elif L["op"] == "maxpool":
            attrs = [attr_ints("kernel_shape", [L["kh"], L["kw"]], packed),
                     attr_ints("strides", [L["stride"]] * 2, packed), attr_ints("pads", [L["pad"]] * 4, packed)]
            nodes.append(node("MaxPool", [x], [t], attrs))
        elif L["op"] == "gavgpool":
            nodes.append(node("GlobalAveragePool", [x], [t]))
        elif L["op"] == "fc":
            if not flat:
                nodes.append(node("Flatten", [x], [t + "_flat"], [attr_int("axis", 1)]))
                x = t + "_flat"
                flat = True
            W = weights[i].astype(np.float32).reshape(oc, h, w, c).transpose(0, 3, 1, 2).reshape(oc, h * w * c)
            inits += [tensor("w%d" % i, W), tensor("b%d" % i, biases[i].astype(np.float32))]
            nodes.append(node("Gemm", [x, "w%d" % i, "b%d" % i], [t], [attr_int("transB", 1)]))
        else:
            raise ValueError(L["op"])
        if L["residual_from"] >= 0:
            nodes.append(node("Add", [t, out_name[L["residual_from"]]], [t + "_sum"]))
            t = t + "_sum"
        if L["act"] == "relu":
            nodes.append(node("Relu", [t], [t + "_act"]))
            t = t + "_act"
        elif L["act"] == "relu6":
            if clip_as_inputs:
                nodes.append(node("Clip", [t, "clip_lo", "clip_hi"], [t + "_act"]))
            else:
                nodes.append(node("Clip", [t], [t + "_act"], [attr_float("min", 0.0), attr_float("max", 6.0)]))
            t = t + "_act"
        out_name[i] = t
        cur = t
    last = shapes[-1][1]
    inputs = [value_info("input", [batch, net["in_c"], net["in_h"], net["in_w"]])]
    outputs = [value_info(cur, [batch, last[2]] if flat else [batch, last[2], last[0], last[1]])]
    return model(nodes, inits, inputs, outputs, opset=13 if clip_as_inputs else 6)
