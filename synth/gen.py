"""Seeded synthetic tensors for the CNN workloads (inputs, weights, biases).

One master seed drives a NumPy PCG64 generator; the draw order is: network input, then for every
layer in list order its weight and then its bias.  Input and weights are drawn in fp32 and rounded
once to fp16 (round-to-nearest-even); biases stay fp32.  The same bits are handed to every
consumer, so no consumer needs to repeat any arithmetic of the method.

Recipe: inputs ~U(-1,1) or ~N(0,1) as the workload states, weights ~N(0, sqrt(2/fan_in))
(fan_in = kh*kw*cin/groups), biases ~U(-0.1,0.1).  The last convolution of a residual branch
(the one that carries `residual_from`) is scaled by `RESIDUAL_BRANCH_GAIN` so that activations of
deep residual stacks stay inside the fp16 range, playing the role of a small folded batch-norm
scale.
"""
import numpy as np

MASTER_SEED = 201105630
RESIDUAL_BRANCH_GAIN = 0.25


def weight_shape(L):
    if L["op"] == "conv":
        return (L["cout"], L["kh"], L["kw"], L["cin"])
    if L["op"] == "dwconv":
        return (L["cout"], L["kh"], L["kw"], 1)
    if L["op"] == "fc":
        return (L["cout"], 1, 1, L["cin"])
    return None


def make_params(net, batch, seed=MASTER_SEED, residual_gain=RESIDUAL_BRANCH_GAIN):
    """Returns (x, weights, biases): x fp16 [batch,H,W,C]; weights[i] fp16 or None; biases[i]
    fp32 or None.  residual_gain scales the weights of layers that add a residual (1.0 = plain
    He-normal)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    shape = (batch, net["in_h"], net["in_w"], net["in_c"])
    if net.get("input_dist", "normal") == "uniform":
        x = rng.uniform(-1.0, 1.0, size=shape).astype(np.float32)
    else:
        x = rng.standard_normal(size=shape, dtype=np.float32)
    x = x.astype(np.float16)
    weights, biases = [], []
    for L in net["layers"]:
        ws = weight_shape(L)
        if ws is None:
            weights.append(None)
            biases.append(None)
            continue
        fan_in = ws[1] * ws[2] * ws[3]
        std = np.float32(np.sqrt(2.0 / fan_in))
        if L["residual_from"] >= 0:
            std = np.float32(std * residual_gain)
        w = rng.standard_normal(size=ws, dtype=np.float32) * std
        weights.append(w.astype(np.float16))
        if L["has_bias"]:
            biases.append(rng.uniform(-0.1, 0.1, size=(L["cout"],)).astype(np.float32))
        else:
            biases.append(None)
    return x, weights, biases


VGG16_BODY = [  # VGG-16's convolutions behind its first layer: (cin, cout, a 2x2 max pool follows), input 64 channels
    (64, 64, True), (64, 128, False), (128, 128, True), (128, 256, False), (256, 256, False), (256, 256, True),
    (256, 512, False), (512, 512, False), (512, 512, True), (512, 512, False), (512, 512, False), (512, 512, True)]


def make_i8_chain(batch, hw, specs=VGG16_BODY, seed=MASTER_SEED):
    """Seeded operands of a chain of quantised 3x3 layers (ReLU behind each): (x int8 [batch,hw,hw,cin0],
    [(weight, scale, bias, pool), ...]); each layer drawn by make_i8_layer with its own seed."""
    x = make_i8_layer(batch, hw, hw, specs[0][0], 16, 3, seed)[0]
    return x, [make_i8_layer(1, 1, 1, ci, co, 3, seed + 1 + i)[1:] + (pool,) for i, (ci, co, pool) in enumerate(specs)]


def make_i8_layer(batch, h, w, cin, cout, k=3, seed=MASTER_SEED, full_range=False):
    """Seeded operands of one quantised convolution layer: (x int8 [batch,h,w,cin], weight int8
    [cout,k,k,cin], scale fp32 [cout], bias fp32 [cout]).

    Recipe: activations round(16 * N(0,1)) and weights round(24 * N(0,1)), clipped to [-127, 127]
    (`full_range`: both uniform over [-128, 127], the largest accumulators the format allows);
    the per-channel scale brings the accumulator's spread (sqrt(k*k*cin) * 16 * 24) to about 48
    output steps, times U(0.5, 1.5), so that outputs use the int8 range and a few per cent
    saturate; bias ~U(-8, 8)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    if full_range:
        x = rng.integers(-128, 128, size=(batch, h, w, cin), dtype=np.int64).astype(np.int8)
        wt = rng.integers(-128, 128, size=(cout, k, k, cin), dtype=np.int64).astype(np.int8)
        spread = np.sqrt(k * k * cin) * 74.0 * 74.0
    else:
        x = np.clip(np.rint(rng.standard_normal(size=(batch, h, w, cin), dtype=np.float32) * 16.0),
                    -127, 127).astype(np.int8)
        wt = np.clip(np.rint(rng.standard_normal(size=(cout, k, k, cin), dtype=np.float32) * 24.0),
                     -127, 127).astype(np.int8)
        spread = np.sqrt(k * k * cin) * 16.0 * 24.0
    scale = (48.0 / spread * rng.uniform(0.5, 1.5, size=(cout,))).astype(np.float32)
    bias = rng.uniform(-8.0, 8.0, size=(cout,)).astype(np.float32)
    return x, wt, scale, bias
