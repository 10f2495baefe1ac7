"""Python face of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this module; the GPU
library never does, and nothing here imports the GPU library.  Each layer function forwards to
the plain nested-loop C routine of the same name in dlf_oracle.c; `run_net` applies them layer by
layer, unfused, which is the definition the fused execution must be equivalent to (paper, Sec. I:
fusion rewrites the computation without changing its result; Sec. III-B: fusion only changes
where intermediates live).

Pins (tests/test_oracle_*.py): tap-count closed form, delta/shift kernels, linearity, 1x1 conv and
FC against numpy.matmul, single-channel conv against scipy.signal.correlate2d, stride-2 against
subsampled stride-1, depthwise against per-channel correlate2d, pooling against reshape/max and
mean, hand-computed values, and tile-wise fused == whole-layer unfused bit equality.  The quantised
convolution (tests/test_oracle_i8.py): accumulators against the fp64 convolution above, numpy
integer matmul and scipy correlate2d; the requantisation against exact rational arithmetic on
hand-made ties, saturation and a case where a two-rounding multiply-add would differ.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None
_F = ctypes.POINTER(ctypes.c_float)
ACT_CODE = {"none": 0, "relu": 1, "relu6": 2}


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(_build.build())
        i = ctypes.c_int
        for sfx in ("f32", "f64"):
            getattr(_lib, "orc_conv2d_" + sfx).argtypes = [_F, i, i, i, i, _F, _F, i, i, i, i, i,
                                                           i, _F]
            getattr(_lib, "orc_fc_" + sfx).argtypes = [_F, i, i, _F, _F, i, _F]
            getattr(_lib, "orc_global_avgpool_" + sfx).argtypes = [_F, i, i, i, i, _F]
        _I8 = ctypes.POINTER(ctypes.c_int8)
        _lib.orc_conv2d_i8.argtypes = [_I8, i, i, i, i, _I8, _F, _F, i, i, i, i, i, i, _I8,
                                       ctypes.POINTER(ctypes.c_int32)]
        _lib.orc_conv2d_i8.restype = ctypes.c_int
        _lib.orc_maxpool.argtypes = [_F, i, i, i, i, i, i, i, i, _F]
        _lib.orc_add.argtypes = [_F, _F, ctypes.c_size_t, _F]
        _lib.orc_act.argtypes = [_F, ctypes.c_size_t, i]
        for name in ("orc_conv2d_f32", "orc_conv2d_f64", "orc_fc_f32", "orc_fc_f64",
                     "orc_global_avgpool_f32", "orc_global_avgpool_f64", "orc_maxpool", "orc_add",
                     "orc_act"):
            getattr(_lib, name).restype = None
    return _lib


def num_threads():
    """Host threads the C loops run on."""
    lib().orc_num_threads.restype = ctypes.c_int
    return int(lib().orc_num_threads())


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _p(a):
    return a.ctypes.data_as(_F) if a is not None else None


def conv2d(x, w, b=None, stride=1, pad=0, groups=1, acc="f32"):
    """x [N,H,W,Cin], w [Cout,Kh,Kw,Cin/groups], b [Cout] or None -> [N,Ho,Wo,Cout] (fp32)."""
    x, w = _f32(x), _f32(w)
    b = _f32(b) if b is not None else None
    N, H, W, Cin = x.shape
    Cout, Kh, Kw, cig = w.shape
    assert cig * groups == Cin and Cout % groups == 0
    Ho = (H + 2 * pad - Kh) // stride + 1
    Wo = (W + 2 * pad - Kw) // stride + 1
    out = np.empty((N, Ho, Wo, Cout), dtype=np.float32)
    getattr(lib(), "orc_conv2d_" + acc)(_p(x), N, H, W, Cin, _p(w), _p(b), Cout, Kh, Kw, stride,
                                        pad, groups, _p(out))
    return out


def conv2d_i8(x, w, scale, bias, stride=1, pad=0, relu=False, return_acc=False):
    """Quantised convolution (see dlf_oracle_i8.c): x int8 [N,H,W,Cin], w int8 [Cout,Kh,Kw,Cin],
    scale / bias fp32 [Cout] -> int8 [N,Ho,Wo,Cout] (and the int32 accumulators on request)."""
    x = np.ascontiguousarray(x, dtype=np.int8)
    w = np.ascontiguousarray(w, dtype=np.int8)
    scale, bias = _f32(scale), _f32(bias)
    N, H, W, Cin = x.shape
    Cout, Kh, Kw, ci = w.shape
    assert ci == Cin and scale.shape == (Cout,) and bias.shape == (Cout,)
    Ho = (H + 2 * pad - Kh) // stride + 1
    Wo = (W + 2 * pad - Kw) // stride + 1
    out = np.empty((N, Ho, Wo, Cout), dtype=np.int8)
    acc = np.empty((N, Ho, Wo, Cout), dtype=np.int32)
    p8 = ctypes.POINTER(ctypes.c_int8)
    rc = lib().orc_conv2d_i8(x.ctypes.data_as(p8), N, H, W, Cin, w.ctypes.data_as(p8), _p(scale),
                             _p(bias), Cout, Kh, Kw, stride, pad, int(bool(relu)),
                             out.ctypes.data_as(p8), acc.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    if rc != 0:
        raise OverflowError("an accumulator left the 32-bit range")
    return (out, acc) if return_acc else out


def maxpool2x2_i8(x):
    """2x2 stride-2 max pool without padding on an int8 map [N,H,W,C] (a last odd row or column is
    dropped): the plain definition, by reshaping."""
    x = np.asarray(x)
    N, H, W, C = x.shape
    return x[:, :H // 2 * 2, :W // 2 * 2].reshape(N, H // 2, 2, W // 2, 2, C).max(axis=(2, 4))


def fc(x, w, b=None, acc="f32"):
    """x [N,K], w [Cout,K] -> [N,Cout] (Eq. 2 with M = batch)."""
    x, w = _f32(x), _f32(w)
    b = _f32(b) if b is not None else None
    N, K = x.shape
    Cout = w.shape[0]
    assert w.shape[1] == K
    out = np.empty((N, Cout), dtype=np.float32)
    getattr(lib(), "orc_fc_" + acc)(_p(x), N, K, _p(w), _p(b), Cout, _p(out))
    return out


def maxpool(x, k, stride, pad=0):
    x = _f32(x)
    N, H, W, C = x.shape
    Ho = (H + 2 * pad - k) // stride + 1
    Wo = (W + 2 * pad - k) // stride + 1
    out = np.empty((N, Ho, Wo, C), dtype=np.float32)
    lib().orc_maxpool(_p(x), N, H, W, C, k, k, stride, pad, _p(out))
    return out


def global_avgpool(x, acc="f32"):
    x = _f32(x)
    N, H, W, C = x.shape
    out = np.empty((N, 1, 1, C), dtype=np.float32)
    getattr(lib(), "orc_global_avgpool_" + acc)(_p(x), N, H, W, C, _p(out))
    return out


def add(a, b):
    a, b = _f32(a), _f32(b)
    assert a.shape == b.shape
    out = np.empty_like(a)
    lib().orc_add(_p(a), _p(b), a.size, _p(out))
    return out


def act(x, name):
    """Returns a new array with the activation applied."""
    y = _f32(x).copy()
    lib().orc_act(_p(y), y.size, ACT_CODE[name])
    return y


def round_fp16(x):
    """Round-to-nearest-even to fp16 and back (diagnostic mode for intermediates)."""
    return np.asarray(x, dtype=np.float32).astype(np.float16).astype(np.float32)


def apply_layer(L, x, w, b, residual=None, acc="f32"):
    """One layer of the list, including residual add and activation (act after the add)."""
    op = L["op"]
    if op == "conv":
        y = conv2d(x, w.reshape(L["cout"], L["kh"], L["kw"], L["cin"]), b, L["stride"], L["pad"],
                   1, acc)
    elif op == "dwconv":
        y = conv2d(x, w.reshape(L["cout"], L["kh"], L["kw"], 1), b, L["stride"], L["pad"],
                   L["cin"], acc)
    elif op == "fc":
        n = x.shape[0]
        y = fc(x.reshape(n, -1), w.reshape(L["cout"], L["cin"]), b, acc).reshape(n, 1, 1, -1)
    elif op == "maxpool":
        y = maxpool(x, L["kh"], L["stride"], L["pad"])
    elif op == "gavgpool":
        y = global_avgpool(x, acc)
    else:
        raise ValueError(op)
    if residual is not None:
        y = add(y, residual)
    if L["act"] != "none":
        y = act(y, L["act"])
    return y


def run_net(net, x, weights, biases, acc="f32", round_intermediates=False, keep_all=False,
            first=0, last=None, given=None):
    """Layer-by-layer, unfused forward pass.

    x: [N,H,W,C] (any float dtype; converted to fp32).  weights/biases: per-layer arrays or None.
    round_intermediates: round every layer output to fp16 (what a device that stores fp16
    activations does); default keeps fp32.  `first`/`last` run a sub-range of layers; `given`
    maps layer index -> output array for tensors produced outside that range (index -1 = net
    input).  Returns the last output, or the list of all outputs if keep_all.
    """
    layers = net["layers"]
    n = len(layers)
    last = n - 1 if last is None else last
    outs = dict(given or {})
    if -1 not in outs:
        outs[-1] = _f32(x)
    needed_later = {}
    for i in range(first, last + 1):
        L = layers[i]
        src = i - 1 if L["input_from"] < 0 else L["input_from"]
        needed_later[src] = i
        if L["residual_from"] >= 0:
            needed_later[L["residual_from"]] = i
    for i in range(first, last + 1):
        L = layers[i]
        src = i - 1 if L["input_from"] < 0 else L["input_from"]
        res = outs[L["residual_from"]] if L["residual_from"] >= 0 else None
        w = _f32(weights[i]) if weights[i] is not None else None
        y = apply_layer(L, outs[src], w, biases[i], res, acc)
        if round_intermediates:
            y = round_fp16(y)
        outs[i] = y
        if not keep_all:
            for k in [k for k, lastuse in needed_later.items() if lastuse <= i and k != last]:
                outs.pop(k, None)
                needed_later.pop(k)
    if keep_all:
        return [outs[i] for i in range(first, last + 1)]
    return outs[last]


def fused_conv_tile(layers, x, weights, biases, oy, ox, th, tw, masked=True, acc="f32"):
    """Evaluate output tile [oy:oy+th, ox:ox+tw] of a chain of convolutions from an input halo
    tile only, the way a fused block does (Sec. III-B, Sec. IV-B: the halo of earlier layers is
    recomputed; intermediates never leave the tile).

    Working backwards from the tile gives the region each layer must produce.  Each layer is then
    evaluated with pad = 0 on its input region.  Positions of an intermediate region that lie
    outside the true feature map hold the padding value 0 when `masked` (required for equivalence
    with the layer-by-layer definition); with masked=False they hold whatever the convolution of
    the virtual extension gives, which is the classic fusion mistake and must differ.
    Returns the tile [N, th, tw, Cout].
    """
    x = _f32(x)
    N, H, W, _ = x.shape
    dims = [(H, W)]
    for L in layers:
        h, w_ = dims[-1]
        dims.append(((h + 2 * L["pad"] - L["kh"]) // L["stride"] + 1,
                     (w_ + 2 * L["pad"] - L["kw"]) // L["stride"] + 1))
    # regions[l] = (y0, x0, h, w) of the OUTPUT of layer l-1 (regions[0] = input of layer 0)
    regions = [None] * (len(layers) + 1)
    regions[len(layers)] = (oy, ox, th, tw)
    for l in range(len(layers) - 1, -1, -1):
        L = layers[l]
        y0, x0, h, w_ = regions[l + 1]
        regions[l] = (y0 * L["stride"] - L["pad"], x0 * L["stride"] - L["pad"],
                      (h - 1) * L["stride"] + L["kh"], (w_ - 1) * L["stride"] + L["kw"])

    def crop(t, reg, full_hw):
        y0, x0, h, w_ = reg
        out = np.zeros((t.shape[0], h, w_, t.shape[3]), dtype=np.float32)
        ys, ye = max(y0, 0), min(y0 + h, full_hw[0])
        xs, xe = max(x0, 0), min(x0 + w_, full_hw[1])
        if ys < ye and xs < xe:
            out[:, ys - y0:ye - y0, xs - x0:xe - x0, :] = t[:, ys:ye, xs:xe, :]
        return out

    cur = crop(x, regions[0], dims[0])
    for l, L in enumerate(layers):
        groups = L["cin"] if L["op"] == "dwconv" else 1
        cig = L["cin"] // groups
        w = _f32(weights[l]).reshape(L["cout"], L["kh"], L["kw"], cig)
        y = conv2d(cur, w, biases[l], L["stride"], 0, groups, acc)
        if L["act"] != "none":
            y = act(y, L["act"])
        y0, x0, h, w_ = regions[l + 1]
        assert y.shape[1] == h and y.shape[2] == w_
        if masked:
            fh, fw = dims[l + 1]
            yy = np.arange(y0, y0 + h)
            xx = np.arange(x0, x0 + w_)
            valid = ((yy >= 0) & (yy < fh))[:, None] & ((xx >= 0) & (xx < fw))[None, :]
            y = np.where(valid[None, :, :, None], y, np.float32(0.0))
        cur = y
    return cur
