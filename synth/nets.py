"""Layer lists of the synthetic CNN workloads (shapes only, no arithmetic).

A network is a list of plain dicts, one per layer, in execution order:

    op            'conv' | 'dwconv' | 'fc' | 'maxpool' | 'gavgpool'
    cin, cout     channel counts (pooling: cin == cout)
    kh, kw        kernel size (fc / gavgpool: 1)
    stride, pad   spatial stride and symmetric zero (conv) / -inf (maxpool) padding
    has_bias      1 if a per-output-channel fp32 bias (folded batch-norm shift) is added
    act           'none' | 'relu' | 'relu6'; applied after the residual add if there is one
    input_from    -1 = output of the previous layer (the net input for layer 0),
                  else index of the layer whose output feeds this one
    residual_from -1 = none, else index of the layer whose output is added before `act`

Residual networks are linearised: a bottleneck is  1x1a, 3x3, [projection], 1x1b  where the
projection reads the block input (`input_from`) and 1x1b reads the 3x3 (`input_from`) and adds
the projection or the block input (`residual_from`).

The shapes follow the layer notation {Cin, Cout, Hout x Wout, Hk x Wk} used in Sec. II-B of the
paper and the standard definitions of the evaluated network families (Sec. V, Table
"Networks description").
"""

ACTS = ("none", "relu", "relu6")
OPS = ("conv", "dwconv", "fc", "maxpool", "gavgpool")


def _layer(op, cin, cout, k=1, stride=1, pad=0, bias=1, act="none", input_from=-1,
           residual_from=-1):
    return dict(op=op, cin=int(cin), cout=int(cout), kh=int(k), kw=int(k), stride=int(stride),
                pad=int(pad), has_bias=int(bias), act=act, input_from=int(input_from),
                residual_from=int(residual_from))


def conv(cin, cout, k=3, stride=1, pad=None, act="relu", **kw):
    if pad is None:
        pad = k // 2
    return _layer("conv", cin, cout, k, stride, pad, 1, act, **kw)


def dwconv(c, k=3, stride=1, act="relu6"):
    return _layer("dwconv", c, c, k, stride, k // 2, 1, act)


def fc(cin, cout, act="none"):
    return _layer("fc", cin, cout, 1, 1, 0, 1, act)


def maxpool(c, k=2, stride=2, pad=0):
    return _layer("maxpool", c, c, k, stride, pad, 0, "none")


def gavgpool(c):
    return _layer("gavgpool", c, c, 1, 1, 0, 0, "none")


def conv_chain(c, depth, act="relu"):
    """`depth` identical {C, C, HxW, 3x3} stride-1 pad-1 convolutions (Sec. III-B sweep)."""
    return [conv(c, c, 3, 1, 1, act) for _ in range(depth)]


def two_layer_block():
    """Config 1: two 16->16 3x3 convolutions with bias and ReLU on a 32x32x16 input."""
    return dict(name="block2", layers=conv_chain(16, 2), in_h=32, in_w=32, in_c=16,
                input_dist="uniform")


def chain4(c, hw=56):
    """Config 2: four C->C 3x3 convolutions with bias and ReLU at hw x hw."""
    return dict(name=f"chain4_c{c}", layers=conv_chain(c, 4), in_h=hw, in_w=hw, in_c=c,
                input_dist="uniform")


def identical_chain(c, hw, depth):
    """Sec. III-B / IV-B style model of `depth` identical 3x3 convolutions."""
    return dict(name=f"chain{depth}_c{c}_{hw}", layers=conv_chain(c, depth), in_h=hw, in_w=hw,
                in_c=c, input_dist="uniform")


def vgg(widths_per_stage, name, in_hw=224, with_fc=True):
    layers = []
    cin = 3
    for stage in widths_per_stage:
        for cout in stage:
            layers.append(conv(cin, cout, 3, 1, 1, "relu"))
            cin = cout
        layers.append(maxpool(cin, 2, 2, 0))
    if with_fc:
        hw = in_hw // (2 ** len(widths_per_stage))
        layers.append(fc(hw * hw * cin, 4096, "relu"))
        layers.append(fc(4096, 4096, "relu"))
        layers.append(fc(4096, 1000, "none"))
    return dict(name=name, layers=layers, in_h=in_hw, in_w=in_hw, in_c=3, input_dist="normal")


def vgg16(in_hw=224, with_fc=True):
    """Config 3: 13 conv3x3 + 5 maxpool + 3 FC."""
    return vgg([[64, 64], [128, 128], [256] * 3, [512] * 3, [512] * 3], "vgg16", in_hw, with_fc)


def vgg19(in_hw=224, with_fc=True):
    return vgg([[64, 64], [128, 128], [256] * 4, [512] * 4, [512] * 4], "vgg19", in_hw, with_fc)


def _bottleneck(layers, cin, width, stride, project):
    """Append one bottleneck; returns the index of its last layer. Stride sits on the 3x3."""
    block_in = len(layers) - 1          # index of the layer producing the block input
    cout = 4 * width
    layers.append(conv(cin, width, 1, 1, 0, "relu", input_from=-1))
    layers.append(conv(width, width, 3, stride, 1, "relu"))
    i3 = len(layers) - 1
    if project:
        layers.append(conv(cin, cout, 1, stride, 0, "none", input_from=block_in))
        res = len(layers) - 1
        layers.append(conv(width, cout, 1, 1, 0, "relu", input_from=i3, residual_from=res))
    else:
        layers.append(conv(width, cout, 1, 1, 0, "relu", residual_from=block_in))
    return len(layers) - 1


def _basic_block(layers, cin, width, stride, project):
    block_in = len(layers) - 1
    layers.append(conv(cin, width, 3, stride, 1, "relu"))
    i1 = len(layers) - 1
    if project:
        layers.append(conv(cin, width, 1, stride, 0, "none", input_from=block_in))
        res = len(layers) - 1
        layers.append(conv(width, width, 3, 1, 1, "relu", input_from=i1, residual_from=res))
    else:
        layers.append(conv(width, width, 3, 1, 1, "relu", residual_from=block_in))
    return len(layers) - 1


def resnet(blocks, bottleneck, name, in_hw=224, with_head=True):
    layers = [conv(3, 64, 7, 2, 3, "relu"), maxpool(64, 3, 2, 1)]
    cin = 64
    for stage, nblk in enumerate(blocks):
        width = 64 << stage
        for b in range(nblk):
            stride = 2 if (b == 0 and stage > 0) else 1
            if bottleneck:
                project = (b == 0)
                _bottleneck(layers, cin, width, stride, project)
                cin = 4 * width
            else:
                project = (b == 0 and stage > 0)
                _basic_block(layers, cin, width, stride, project)
                cin = width
    if with_head:
        layers.append(gavgpool(cin))
        layers.append(fc(cin, 1000, "none"))
    return dict(name=name, layers=layers, in_h=in_hw, in_w=in_hw, in_c=3, input_dist="normal")


def resnet50(in_hw=224, with_head=True):
    """Config 4: bottleneck stages [3,4,6,3], projection shortcut in each stage's first block."""
    return resnet([3, 4, 6, 3], True, "resnet50", in_hw, with_head)


def resnet18(in_hw=224, with_head=True):
    return resnet([2, 2, 2, 2], False, "resnet18", in_hw, with_head)


def alexnet(in_hw=224):
    """Single-tower 64-192-384-256-256 variant (convolutions and pools only, plus 3 FC)."""
    layers = [conv(3, 64, 11, 4, 2, "relu"), maxpool(64, 3, 2, 0),
              conv(64, 192, 5, 1, 2, "relu"), maxpool(192, 3, 2, 0),
              conv(192, 384, 3, 1, 1, "relu"), conv(384, 256, 3, 1, 1, "relu"),
              conv(256, 256, 3, 1, 1, "relu"), maxpool(256, 3, 2, 0),
              fc(6 * 6 * 256, 4096, "relu"), fc(4096, 4096, "relu"), fc(4096, 1000, "none")]
    return dict(name="alexnet", layers=layers, in_h=in_hw, in_w=in_hw, in_c=3,
                input_dist="normal")


MOBILENET_V1 = [(64, 1), (128, 2), (128, 1), (256, 2), (256, 1), (512, 2),
                (512, 1), (512, 1), (512, 1), (512, 1), (512, 1), (1024, 2), (1024, 1)]


def mobilenet_v1(in_hw=224, with_head=True, nblocks=13):
    """Config 5: conv3x3 s2 32, then depthwise 3x3 + pointwise 1x1 blocks, ReLU6 everywhere."""
    layers = [conv(3, 32, 3, 2, 1, "relu6")]
    cin = 32
    for cout, stride in MOBILENET_V1[:nblocks]:
        layers.append(dwconv(cin, 3, stride, "relu6"))
        layers.append(conv(cin, cout, 1, 1, 0, "relu6"))
        cin = cout
    if with_head:
        layers.append(gavgpool(cin))
        layers.append(fc(cin, 1000, "none"))
    return dict(name="mobilenet_v1", layers=layers, in_h=in_hw, in_w=in_hw, in_c=3,
                input_dist="normal")


def infer_shapes(net):
    """Per-layer (H, W, C) input and output shapes; plain integer shape inference."""
    shapes_out = []
    res = []
    for i, L in enumerate(net["layers"]):
        src = L["input_from"]
        if src < 0:
            hin = (net["in_h"], net["in_w"], net["in_c"]) if i == 0 else shapes_out[i - 1]
        else:
            hin = shapes_out[src]
        h, w, c = hin
        if L["op"] in ("conv", "dwconv", "maxpool"):
            assert c == L["cin"], (i, c, L)
            ho = (h + 2 * L["pad"] - L["kh"]) // L["stride"] + 1
            wo = (w + 2 * L["pad"] - L["kw"]) // L["stride"] + 1
            out = (ho, wo, L["cout"])
        elif L["op"] == "gavgpool":
            out = (1, 1, c)
        elif L["op"] == "fc":
            assert h * w * c == L["cin"], (i, hin, L)
            out = (1, 1, L["cout"])
        else:
            raise ValueError(L["op"])
        shapes_out.append(out)
        res.append((hin, out))
    return res
