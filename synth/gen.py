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
