"""ONNX front end: a model file -> the layer list and parameter arrays `dlf_net_create` takes.

Algorithm 1 takes an ONNX file as its input, and the tool chain of Sec. IV-C ("DLFusion Compiler
Tool Chain") turns it into per-layer specifications before the optimizer runs; this module is that
step for the operators the CNN families of Sec. V consist of:

    Conv (group 1, or depthwise: group = Cin = Cout), BatchNormalization (folded into the
    convolution in front of it), Relu, Clip(0, 6), MaxPool, GlobalAveragePool / whole-map
    AveragePool, Add (residual), Flatten / Reshape / Squeeze in front of a fully connected layer,
    Gemm, MatMul (+ Add of a bias vector).

No ONNX or protobuf package is needed: the file is read with a small decoder of the protobuf wire
format (varint, 64-bit, length-delimited and 32-bit fields) and the field numbers of the ONNX
schema (ModelProto, GraphProto, NodeProto, AttributeProto, TensorProto, ValueInfoProto).

What comes out is a description, no arithmetic of the method: layers in the graph's (topological)
order with `input_from` / `residual_from` links, weights re-laid from ONNX's [Cout][Cin][kh][kw] to
the library's [Cout][kh][kw][Cin] and rounded to fp16, biases in fp32.  Activations of the library
are NHWC; the declared NCHW input shape is read for H, W and C only, and a fully connected layer
behind a feature map gets its columns permuted from ONNX's (c, h, w) flattening to (h, w, c).
"""
import struct

import numpy as np


class OnnxIngestError(ValueError):
    pass


# ---------------------------------------------------------------- protobuf wire format

def _varint(buf, pos):
    result = 0
    shift = 0
    while True:
        if pos >= len(buf):
            raise OnnxIngestError("truncated varint")
        b = buf[pos]
        pos += 1
        result |= (b & 0x7F) << shift
        if not b & 0x80:
            return result, pos
        shift += 7
        if shift > 63:
            raise OnnxIngestError("varint longer than 64 bits")


def _signed64(v):
    return v - (1 << 64) if v >= (1 << 63) else v


def _fields(buf):
    """Yields (field number, wire type, value) of one message: int for varint / fixed fields, a
    memoryview for length-delimited ones."""
    buf = memoryview(buf)
    pos = 0
    n = len(buf)
    while pos < n:
        key, pos = _varint(buf, pos)
        field, wt = key >> 3, key & 7
        if wt == 0:
            val, pos = _varint(buf, pos)
        elif wt == 1:
            if pos + 8 > n:
                raise OnnxIngestError("truncated 64-bit field")
            val = struct.unpack_from("<Q", buf, pos)[0]
            pos += 8
        elif wt == 2:
            ln, pos = _varint(buf, pos)
            if pos + ln > n:
                raise OnnxIngestError("truncated length-delimited field")
            val = buf[pos:pos + ln]
            pos += ln
        elif wt == 5:
            if pos + 4 > n:
                raise OnnxIngestError("truncated 32-bit field")
            val = struct.unpack_from("<I", buf, pos)[0]
            pos += 4
        else:
            raise OnnxIngestError("unsupported wire type %d" % wt)
        yield field, wt, val


def _packed_varints(val, wt):
    """A repeated integer field arrives packed (one length-delimited blob) or one value per key."""
    if wt == 0:
        return [_signed64(val)]
    out = []
    pos = 0
    while pos < len(val):
        v, pos = _varint(val, pos)
        out.append(_signed64(v))
    return out


def _packed_fixed32(val, wt):
    if wt == 5:
        return [struct.unpack("<f", struct.pack("<I", val))[0]]
    return list(np.frombuffer(bytes(val), dtype="<f4"))


# ---------------------------------------------------------------- ONNX messages

_DTYPES = {1: np.dtype("<f4"), 2: np.dtype("u1"), 3: np.dtype("i1"), 6: np.dtype("<i4"),
           7: np.dtype("<i8"), 10: np.dtype("<f2"), 11: np.dtype("<f8")}


def _parse_tensor(buf):
    dims, dtype, name, raw = [], 0, "", None
    floats, int32s, int64s, doubles = [], [], [], []
    for f, wt, v in _fields(buf):
        if f == 1:
            dims += _packed_varints(v, wt)
        elif f == 2:
            dtype = v
        elif f == 4:
            floats += _packed_fixed32(v, wt)
        elif f == 5:
            int32s += _packed_varints(v, wt)
        elif f == 7:
            int64s += _packed_varints(v, wt)
        elif f == 8:
            name = bytes(v).decode("utf-8")
        elif f == 9:
            raw = bytes(v)
        elif f == 10:
            doubles += list(np.frombuffer(bytes(v), dtype="<f8")) if wt == 2 else \
                [struct.unpack("<d", struct.pack("<Q", v))[0]]
        elif f == 14 and v != 0:
            raise OnnxIngestError("tensor %r keeps its data in an external file" % name)
    if dtype not in _DTYPES:
        raise OnnxIngestError("tensor %r: element type %d is not supported" % (name, dtype))
    dt = _DTYPES[dtype]
    if raw is not None:
        arr = np.frombuffer(raw, dtype=dt)
    elif dtype == 1:
        arr = np.asarray(floats, dtype=np.float32)
    elif dtype == 11:
        arr = np.asarray(doubles, dtype=np.float64)
    elif dtype == 7:
        arr = np.asarray(int64s, dtype=np.int64)
    elif dtype == 10:            # fp16 bit patterns travel in int32_data
        arr = np.asarray(int32s, dtype=np.int64).astype(np.uint16).view(np.float16)
    else:
        arr = np.asarray(int32s, dtype=np.int64).astype(dt)
    count = int(np.prod(dims)) if dims else 1
    if arr.size != count:
        raise OnnxIngestError("tensor %r: %d values for shape %r" % (name, arr.size, dims))
    return name, arr.reshape(dims)


def _parse_attribute(buf):
    name, out = "", None
    ints, floats = [], []
    has_ints = has_floats = False
    for f, wt, v in _fields(buf):
        if f == 1:
            name = bytes(v).decode("utf-8")
        elif f == 2:
            out = struct.unpack("<f", struct.pack("<I", v))[0]
        elif f == 3:
            out = _signed64(v)
        elif f == 4:
            out = bytes(v)
        elif f == 5:
            out = _parse_tensor(v)[1]
        elif f == 7:
            floats += _packed_fixed32(v, wt)
            has_floats = True
        elif f == 8:
            ints += _packed_varints(v, wt)
            has_ints = True
    if has_ints:
        out = ints
    elif has_floats:
        out = floats
    return name, out


def _parse_node(buf):
    node = dict(inputs=[], outputs=[], name="", op="", attrs={}, domain="")
    for f, wt, v in _fields(buf):
        if f == 1:
            node["inputs"].append(bytes(v).decode("utf-8"))
        elif f == 2:
            node["outputs"].append(bytes(v).decode("utf-8"))
        elif f == 3:
            node["name"] = bytes(v).decode("utf-8")
        elif f == 4:
            node["op"] = bytes(v).decode("utf-8")
        elif f == 5:
            k, a = _parse_attribute(v)
            node["attrs"][k] = a
        elif f == 7:
            node["domain"] = bytes(v).decode("utf-8")
    return node


def _parse_value_info(buf):
    name, shape = "", None
    for f, wt, v in _fields(buf):
        if f == 1:
            name = bytes(v).decode("utf-8")
        elif f == 2:                                       # TypeProto
            for f2, _, v2 in _fields(v):
                if f2 == 1:                                # tensor_type
                    for f3, _, v3 in _fields(v2):
                        if f3 == 2:                        # TensorShapeProto
                            shape = []
                            for f4, _, v4 in _fields(v3):
                                if f4 == 1:                # Dimension
                                    d = None
                                    for f5, _, v5 in _fields(v4):
                                        if f5 == 1:
                                            d = _signed64(v5)
                                    shape.append(d)
    return name, shape


def parse_model(data):
    """-> dict(nodes, initializers {name: array}, inputs [(name, shape)], outputs [...], opset)."""
    graph = None
    opset = 0
    for f, wt, v in _fields(data):
        if f == 7:
            graph = v
        elif f == 8:
            dom, ver = "", 0
            for f2, _, v2 in _fields(v):
                if f2 == 1:
                    dom = bytes(v2).decode("utf-8")
                elif f2 == 2:
                    ver = v2
            if dom in ("", "ai.onnx"):
                opset = ver
    if graph is None:
        raise OnnxIngestError("no graph in the model")
    g = dict(nodes=[], initializers={}, inputs=[], outputs=[], opset=opset)
    for f, wt, v in _fields(graph):
        if f == 1:
            g["nodes"].append(_parse_node(v))
        elif f == 5:
            name, arr = _parse_tensor(v)
            g["initializers"][name] = arr
        elif f == 11:
            g["inputs"].append(_parse_value_info(v))
        elif f == 12:
            g["outputs"].append(_parse_value_info(v))
    return g


# ---------------------------------------------------------------- graph -> layer list

def _layer(op, cin, cout, k, stride, pad, bias, act, input_from):
    return dict(op=op, cin=int(cin), cout=int(cout), kh=int(k), kw=int(k), stride=int(stride),
                pad=int(pad), has_bias=int(bias), act=act, input_from=int(input_from),
                residual_from=-1)


def _square(vals, what, node):
    vals = list(vals)
    if any(v != vals[0] for v in vals):
        raise OnnxIngestError("%s %r: %s %r is not the same in every direction"
                              % (node["op"], node["name"], what, vals))
    return int(vals[0])


class _Builder:
    def __init__(self, g):
        self.g = g
        self.init = g["initializers"]
        self.layers, self.weights, self.biases = [], [], []
        self.shape = []          # (h, w, c) of every layer's output
        self.src = {}            # tensor name -> (layer index or -1 for the net input, flattened?)
        self.uses = {}
        for n in g["nodes"]:
            for t in n["inputs"]:
                self.uses[t] = self.uses.get(t, 0) + 1
        for name, _ in g["outputs"]:
            self.uses[name] = self.uses.get(name, 0) + 1

    def out_shape(self, idx):
        return self.in_shape if idx < 0 else self.shape[idx]

    def link(self, idx):
        """input_from value for a layer appended now whose input is layer idx's output."""
        cur = len(self.layers)
        if idx == cur - 1:
            return -1
        if idx < 0:
            raise OnnxIngestError("only the first layer may read the network input")
        return idx

    def lookup(self, name, node):
        if name not in self.src:
            raise OnnxIngestError("%s %r reads %r, which no supported node produces"
                                  % (node["op"], node["name"], name))
        return self.src[name]

    def const(self, name, node):
        if name not in self.init:
            raise OnnxIngestError("%s %r: operand %r must be an initializer" % (node["op"], node["name"], name))
        return self.init[name]

    def sole_use(self, name):
        return self.uses.get(name, 0) == 1

    def append(self, layer, w, b, shape):
        self.layers.append(layer)
        self.weights.append(None if w is None else np.ascontiguousarray(w.astype(np.float16)))
        self.biases.append(None if b is None else np.ascontiguousarray(b.astype(np.float32)))
        self.shape.append(shape)
        return len(self.layers) - 1

    # ---- operators
    def conv(self, n):
        idx, flat = self.lookup(n["inputs"][0], n)
        h, w_, c = self.out_shape(idx)
        W = self.const(n["inputs"][1], n).astype(np.float32)
        if W.ndim != 4:
            raise OnnxIngestError("Conv %r: only 2-D convolutions" % n["name"])
        cout, cin_g, kh, kw = W.shape
        a = n["attrs"]
        k = _square([kh, kw], "kernel", n)
        stride = _square(a.get("strides", [1, 1]), "stride", n)
        if _square(a.get("dilations", [1, 1]), "dilation", n) != 1:
            raise OnnxIngestError("Conv %r: dilation is not supported" % n["name"])
        auto = a.get("auto_pad", b"NOTSET")
        if auto in (b"NOTSET", b""):
            pad = _square(a.get("pads", [0, 0, 0, 0]), "padding", n)
        elif auto in (b"SAME_UPPER", b"SAME_LOWER") and stride == 1 and k % 2 == 1:
            pad = k // 2
        elif auto == b"VALID":
            pad = 0
        else:
            raise OnnxIngestError("Conv %r: auto_pad %r with stride %d" % (n["name"], auto, stride))
        group = int(a.get("group", 1))
        if group == 1 and cin_g == c:
            op, wl = "conv", W.transpose(0, 2, 3, 1)
        elif group == c and cout == c and cin_g == 1:
            op, wl = "dwconv", W.transpose(0, 2, 3, 1)
        else:
            raise OnnxIngestError("Conv %r: group %d with %d -> %d channels" % (n["name"], group, c, cout))
        bias = self.const(n["inputs"][2], n).astype(np.float32) if len(n["inputs"]) > 2 and n["inputs"][2] \
            else np.zeros(cout, np.float32)
        oh = (h + 2 * pad - k) // stride + 1
        ow = (w_ + 2 * pad - k) // stride + 1
        L = _layer(op, c, cout, k, stride, pad, 1, "none", self.link(idx))
        self.src[n["outputs"][0]] = (self.append(L, wl, bias, (oh, ow, cout)), False)

    def batchnorm(self, n):
        idx, _ = self.lookup(n["inputs"][0], n)
        if idx < 0 or self.layers[idx]["op"] not in ("conv", "dwconv") or not self.sole_use(n["inputs"][0]) \
                or self.layers[idx]["act"] != "none" or self.layers[idx]["residual_from"] >= 0:
            raise OnnxIngestError("BatchNormalization %r does not directly follow a convolution" % n["name"])
        scale, shift, mean, var = (self.const(t, n).astype(np.float64) for t in n["inputs"][1:5])
        eps = float(n["attrs"].get("epsilon", 1e-5))
        g = scale / np.sqrt(var + eps)
        # conv, then (y - mean) g + shift  ==  conv with weights w g and bias (b - mean) g + shift
        w = self.weights[idx].astype(np.float64) * g[:, None, None, None]
        b = (self.biases[idx].astype(np.float64) - mean) * g + shift
        self.weights[idx] = np.ascontiguousarray(w.astype(np.float16))
        self.biases[idx] = np.ascontiguousarray(b.astype(np.float32))
        self.src[n["outputs"][0]] = (idx, False)

    def activation(self, n, act):
        idx, flat = self.lookup(n["inputs"][0], n)
        if idx < 0 or self.layers[idx]["op"] not in ("conv", "dwconv", "fc") or self.layers[idx]["act"] != "none" \
                or not self.sole_use(n["inputs"][0]):
            raise OnnxIngestError("%s %r does not directly follow a convolution, a fully connected "
                                  "layer or a residual add" % (n["op"], n["name"]))
        self.layers[idx]["act"] = act
        self.src[n["outputs"][0]] = (idx, flat)

    def clip(self, n):
        a = n["attrs"]
        lo = a.get("min")
        hi = a.get("max")
        if len(n["inputs"]) > 1 and n["inputs"][1]:
            lo = float(self.const(n["inputs"][1], n).reshape(-1)[0])
        if len(n["inputs"]) > 2 and n["inputs"][2]:
            hi = float(self.const(n["inputs"][2], n).reshape(-1)[0])
        if lo != 0.0 or hi != 6.0:
            raise OnnxIngestError("Clip %r: only the range [0, 6] (ReLU6)" % n["name"])
        self.activation(n, "relu6")

    def pool_geometry(self, n):
        a = n["attrs"]
        k = _square(a["kernel_shape"], "kernel", n)
        stride = _square(a.get("strides", [1, 1]), "stride", n)
        pad = _square(a.get("pads", [0, 0, 0, 0]), "padding", n)
        if int(a.get("ceil_mode", 0)) != 0:
            raise OnnxIngestError("%s %r: ceil_mode" % (n["op"], n["name"]))
        return k, stride, pad

    def maxpool(self, n):
        idx, _ = self.lookup(n["inputs"][0], n)
        h, w_, c = self.out_shape(idx)
        k, stride, pad = self.pool_geometry(n)
        L = _layer("maxpool", c, c, k, stride, pad, 0, "none", self.link(idx))
        shape = ((h + 2 * pad - k) // stride + 1, (w_ + 2 * pad - k) // stride + 1, c)
        self.src[n["outputs"][0]] = (self.append(L, None, None, shape), False)

    def gavgpool(self, n):
        idx, _ = self.lookup(n["inputs"][0], n)
        h, w_, c = self.out_shape(idx)
        if n["op"] == "AveragePool":
            k, stride, pad = self.pool_geometry(n)
            if k != h or k != w_ or pad != 0:
                raise OnnxIngestError("AveragePool %r: only a window that covers the whole map" % n["name"])
        L = _layer("gavgpool", c, c, 1, 1, 0, 0, "none", self.link(idx))
        self.src[n["outputs"][0]] = (self.append(L, None, None, (1, 1, c)), False)

    def add(self, n):
        a, b = n["inputs"][:2]
        if a in self.init or b in self.init:               # bias of a MatMul
            t, v = (b, a) if a in self.init else (a, b)
            idx, flat = self.lookup(t, n)
            if idx < 0 or self.layers[idx]["op"] != "fc" or self.layers[idx]["act"] != "none" or not self.sole_use(t):
                raise OnnxIngestError("Add %r of a constant does not follow a MatMul" % n["name"])
            self.biases[idx] = np.ascontiguousarray(
                (self.biases[idx] + self.init[v].astype(np.float32).reshape(-1)).astype(np.float32))
            self.src[n["outputs"][0]] = (idx, flat)
            return
        ia, _ = self.lookup(a, n)
        ib, _ = self.lookup(b, n)

        def branch_end(i, t):      # a convolution whose bare output only this Add reads
            return i >= 0 and self.layers[i]["op"] == "conv" and self.layers[i]["act"] == "none" \
                and self.layers[i]["residual_from"] < 0 and self.sole_use(t)
        # the later of the two is the end of the residual branch, the earlier one the skip operand
        if ia > ib and branch_end(ia, a):
            end, skip = ia, ib
        elif ib > ia and branch_end(ib, b):
            end, skip = ib, ia
        else:
            raise OnnxIngestError("Add %r: neither operand is the bare output of a later convolution" % n["name"])
        if skip < 0:
            raise OnnxIngestError("Add %r: the network input as a residual operand" % n["name"])
        if self.out_shape(skip) != self.out_shape(end):
            raise OnnxIngestError("Add %r: operand shapes differ" % n["name"])
        self.layers[end]["residual_from"] = skip
        self.src[n["outputs"][0]] = (end, False)

    def reshape(self, n):
        idx, _ = self.lookup(n["inputs"][0], n)
        self.src[n["outputs"][0]] = (idx, True)

    def fully_connected(self, n):
        idx, flat = self.lookup(n["inputs"][0], n)
        h, w_, c = self.out_shape(idx)
        B = self.const(n["inputs"][1], n).astype(np.float32)
        a = n["attrs"]
        if n["op"] == "Gemm":
            if float(a.get("alpha", 1.0)) != 1.0 or float(a.get("beta", 1.0)) != 1.0 or int(a.get("transA", 0)):
                raise OnnxIngestError("Gemm %r: alpha, beta or transA" % n["name"])
            W = B if int(a.get("transB", 0)) else B.T
        else:
            W = B.T
        cout, k = W.shape
        if k != h * w_ * c:
            raise OnnxIngestError("%s %r: %d inputs for a %dx%dx%d map" % (n["op"], n["name"], k, h, w_, c))
        if h * w_ > 1:            # ONNX flattens (c, h, w); the library's activations are (h, w, c)
            W = W.reshape(cout, c, h, w_).transpose(0, 2, 3, 1).reshape(cout, k)
        bias = self.const(n["inputs"][2], n).astype(np.float32).reshape(-1) \
            if n["op"] == "Gemm" and len(n["inputs"]) > 2 and n["inputs"][2] else np.zeros(cout, np.float32)
        L = _layer("fc", k, cout, 1, 1, 0, 1, "none", self.link(idx))
        self.src[n["outputs"][0]] = (self.append(L, W.reshape(cout, 1, 1, k), bias, (1, 1, cout)), True)

    def run(self):
        g = self.g
        net_inputs = [(nm, sh) for nm, sh in g["inputs"] if nm not in self.init]
        if len(net_inputs) != 1:
            raise OnnxIngestError("expected one network input, found %d" % len(net_inputs))
        name, shape = net_inputs[0]
        if shape is None or len(shape) != 4 or any(d is None or d <= 0 for d in shape[1:]):
            raise OnnxIngestError("network input %r needs a declared [N, C, H, W] shape" % name)
        self.in_shape = (int(shape[2]), int(shape[3]), int(shape[1]))
        self.src[name] = (-1, False)
        ops = {"Conv": self.conv, "BatchNormalization": self.batchnorm, "MaxPool": self.maxpool,
               "GlobalAveragePool": self.gavgpool, "AveragePool": self.gavgpool, "Add": self.add,
               "Flatten": self.reshape, "Reshape": self.reshape, "Squeeze": self.reshape,
               "Gemm": self.fully_connected, "MatMul": self.fully_connected, "Clip": self.clip,
               "Relu": lambda n: self.activation(n, "relu"),
               "Identity": lambda n: self.src.__setitem__(n["outputs"][0], self.lookup(n["inputs"][0], n)),
               "Dropout": lambda n: self.src.__setitem__(n["outputs"][0], self.lookup(n["inputs"][0], n))}
        for n in g["nodes"]:
            if n["op"] not in ops or n["domain"] not in ("", "ai.onnx"):
                raise OnnxIngestError("operator %s (node %r) is not supported" % (n["op"], n["name"]))
            ops[n["op"]](n)
        if not self.layers:
            raise OnnxIngestError("the graph holds no layer")
        if len(g["outputs"]) != 1 or self.lookup(g["outputs"][0][0], dict(op="output", name=""))[0] != len(self.layers) - 1:
            raise OnnxIngestError("the graph output must be the last layer's output")
        h, w_, c = self.in_shape
        net = dict(name="onnx", layers=self.layers, in_h=h, in_w=w_, in_c=c, input_dist="normal")
        return net, self.weights, self.biases


def load_onnx(source):
    """source: a path or the bytes of an ONNX model.  -> (net, weights, biases) in the form
    `dlf_net_create` (and the synthetic generators) use: net = dict(layers, in_h, in_w, in_c),
    weights[i] fp16 [Cout][kh][kw][Cin] or None, biases[i] fp32 [Cout] or None."""
    if isinstance(source, (bytes, bytearray, memoryview)):
        data = bytes(source)
    else:
        with open(source, "rb") as f:
            data = f.read()
    return _Builder(parse_model(data)).run()
