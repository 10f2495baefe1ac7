"""The quantised (int8) 3x3 convolution layer of libdlf against the integer oracle, bit for bit:
the library's own choice of kernel shape and tile on maps that span several tiles with ragged
edges and ragged channel blocks, every kernel shape forced, operands over the whole int8 range,
and a chain of four layers each fed the previous one's int8 output."""
import numpy as np
import pytest
import torch

from gpu_util import announce
from synth import gen

pytestmark = pytest.mark.gpu


def _run(x, wt, sc, b, relu, budget=0, pool=False):
    from paper_2011_05630_amd import binding as B
    n, h, w, cin = x.shape
    cout, ksize = wt.shape[0], wt.shape[1]
    layer = B.dlf_i8conv_create(n, h, w, cin, cout, ksize, relu, wt, sc, b, budget, pool)
    if pool:
        h, w = h // 2, w // 2
    try:
        info = B.dlf_i8conv_info(layer)
        xt = torch.from_numpy(x).cuda()
        out = torch.full((n, h, w, cout), 0x55, dtype=torch.int8, device="cuda")
        guard = out.clone()
        B.dlf_i8conv_run(layer, xt.data_ptr(), out.data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        return out.cpu().numpy(), info
    finally:
        B.dlf_i8conv_destroy(layer)


def _check(case, x, wt, sc, b, relu, budget=0, pool=False):
    from oracle import oracle
    announce("i8conv", case, x.shape, "cout", wt.shape[0], "relu", relu, "pool", pool)
    got, info = _run(x, wt, sc, b, relu, budget, pool)
    ref = oracle.conv2d_i8(x, wt, sc, b, 1, wt.shape[1] // 2, relu)
    if pool:
        ref = oracle.maxpool2x2_i8(ref)
    bad = np.argwhere(got != ref)
    assert bad.size == 0, (case, info, len(bad), bad[:5].tolist(),
                           [(int(got[tuple(i)]), int(ref[tuple(i)])) for i in bad[:5]])
    if ref.size >= 4096:
        assert ref.min() <= (0 if relu else (-50 if pool else -100)) and ref.max() >= 100      # the case exercises the range
    return info


CASES = [  # batch, h, w, cin, cout, relu
    (2, 20, 27, 64, 48, False),
    (1, 14, 14, 128, 128, True),
    (3, 9, 33, 64, 80, True),
    (1, 56, 56, 256, 256, True),
    (2, 28, 28, 192, 144, False),
    (1, 7, 7, 512, 512, True),
    (1, 1, 1, 64, 16, False),
]


@pytest.mark.parametrize("case", CASES)
def test_i8conv_equals_oracle(case):
    n, h, w, cin, cout, relu = case
    x, wt, sc, b = gen.make_i8_layer(n, h, w, cin, cout, 3, seed=1000 + h * w + cin)
    _check(case, x, wt, sc, b, relu)


CASES_1X1 = [  # batch, h, w, cin, cout, relu: both block shapes (cout <= 64: 64 x 256), ragged pixel and channel blocks
    (2, 28, 28, 256, 128, True),
    (3, 7, 9, 64, 48, False),
    (1, 56, 56, 64, 256, True),
    (5, 13, 11, 512, 208, False),
    (1, 1, 1, 64, 16, True),
    (2, 14, 14, 1024, 64, True),
]


@pytest.mark.parametrize("case", CASES_1X1)
def test_i8conv_1x1_equals_oracle(case):
    n, h, w, cin, cout, relu = case
    x, wt, sc, b = gen.make_i8_layer(n, h, w, cin, cout, 1, seed=2000 + h * w + cin)
    _check(("1x1",) + case, x, wt, sc, b, relu)


def test_i8conv_1x1_full_range_and_small_budget():
    x, wt, sc, b = gen.make_i8_layer(2, 20, 20, 128, 160, 1, seed=32, full_range=True)
    _check("1x1 full range", x, wt, sc, b, False)
    _check("1x1 full range, 8 CUs (several blocks per workgroup)", x, wt, sc, b, True, budget=8)


@pytest.mark.parametrize("case", [(2, 20, 28, 64, 48, False), (1, 56, 56, 128, 128, True), (3, 9, 33, 64, 80, True),
                                  (1, 14, 14, 512, 512, True), (2, 2, 2, 64, 16, False), (1, 30, 6, 256, 96, True)])
def test_i8conv_with_folded_pool_equals_oracle(case):
    """conv 3x3 + 2x2 max pool as one launch against conv then pool in the oracle; odd maps drop their
    last row / column."""
    n, h, w, cin, cout, relu = case
    x, wt, sc, b = gen.make_i8_layer(n, h, w, cin, cout, 3, seed=4000 + h * w + cin)
    _check(("pool",) + case, x, wt, sc, b, relu, pool=True)


@pytest.mark.parametrize("shape,th,tw", [(0, 8, 16), (1, 14, 14), (2, 16, 28), (3, 14, 28), (4, 16, 32), (4, 14, 28)])
def test_i8conv_with_folded_pool_every_kernel_shape(shape, th, tw):
    from paper_2011_05630_amd import binding as B
    x, wt, sc, b = gen.make_i8_layer(2, 30, 37, 128, 160, 3, seed=60 + shape)
    B.dlf_debug_block3x3_mode(0, shape, th, tw)
    try:
        info = _check(("pool shape", shape, th, tw), x, wt, sc, b, True, budget=64, pool=True)
    finally:
        B.dlf_debug_block3x3_mode(0, -1, 0, 0)
    assert (info["shape"], info["th"], info["tw"]) == (shape, th, tw)


def test_i8conv_full_range_operands():
    x, wt, sc, b = gen.make_i8_layer(2, 12, 18, 128, 96, 3, seed=31, full_range=True)
    x[0, :2] = -128
    wt[:4] = -128                     # the largest products the format allows, accumulators above 2^24
    _check("full range", x, wt, sc, b, False)
    _check("full range relu", x, wt, sc, b, True)


@pytest.mark.parametrize("shape,th,tw,cin", [(0, 8, 16, 64), (1, 14, 14, 128), (2, 16, 28, 64), (3, 14, 28, 128),
                                             (4, 16, 32, 64), (0, 7, 7, 192), (4, 14, 28, 128)])
def test_i8conv_every_kernel_shape(shape, th, tw, cin):
    from paper_2011_05630_amd import binding as B
    x, wt, sc, b = gen.make_i8_layer(2, 30, 37, cin, 160, 3, seed=50 + shape)
    B.dlf_debug_block3x3_mode(0, shape, th, tw)
    try:
        info = _check(("shape", shape, th, tw), x, wt, sc, b, True, budget=64)
    finally:
        B.dlf_debug_block3x3_mode(0, -1, 0, 0)
    assert (info["shape"], info["th"], info["tw"]) == (shape, th, tw)


@pytest.mark.parametrize("k,ksplit,n,h,w,cin,cout", [
    (3, 1, 2, 14, 14, 512, 512), (3, 2, 3, 7, 7, 512, 80), (3, 4, 1, 9, 11, 1024, 272), (3, 2, 2, 13, 5, 512, 48),
    (1, 1, 2, 14, 14, 1024, 256), (1, 2, 5, 7, 7, 2048, 512), (1, 4, 1, 10, 9, 1024, 144), (1, 2, 3, 5, 8, 512, 96), (3, 4, 4, 6, 6, 2048, 64)])
def test_i8conv_small_map_kernel(k, ksplit, n, h, w, cin, cout):
    """The kernel for maps of many channels and few pixels, forced, with K split over 1, 2 and 4 waves
    (integer partial sums: the split changes no bit), ragged tiles and ragged channel slices."""
    from paper_2011_05630_amd import binding as B
    x, wt, sc, b = gen.make_i8_layer(n, h, w, cin, cout, k, seed=300 + ksplit + k + h)
    B.dlf_debug_block3x3_mode(0, 5, ksplit, 0)
    try:
        info = _check(("small map", k, ksplit), x, wt, sc, b, True)
    finally:
        B.dlf_debug_block3x3_mode(0, -1, 0, 0)
    assert info["shape"] == 5 and info["th"] <= 8 and info["tw"] <= 8


@pytest.mark.parametrize("ksplit,n,h,w,cin,cout", [(1, 2, 14, 14, 512, 512), (2, 3, 7, 7, 512, 80), (4, 1, 9, 11, 1024, 272),
                                                   (2, 2, 13, 5, 512, 48), (1, 2, 2, 2, 512, 16), (4, 2, 16, 24, 512, 96),
                                                   (1, 1, 4, 30, 1024, 64)])
def test_i8conv_small_map_kernel_with_folded_pool(ksplit, n, h, w, cin, cout):
    """The small-map kernel with the 2x2 max pool folded in (tiles 8 wide, of even height): one- and
    two-block tiles, ragged tiles, odd maps, K split over 1, 2 and 4 waves."""
    from paper_2011_05630_amd import binding as B
    x, wt, sc, b = gen.make_i8_layer(n, h, w, cin, cout, 3, seed=500 + ksplit + h)
    B.dlf_debug_block3x3_mode(0, 5, ksplit, 0)
    try:
        info = _check(("small map + pool", ksplit), x, wt, sc, b, True, pool=True)
    finally:
        B.dlf_debug_block3x3_mode(0, -1, 0, 0)
    assert info["shape"] == 5 and info["tw"] == 8 and info["th"] % 2 == 0


def test_i8conv_small_map_kernel_is_chosen_where_it_pays():
    from paper_2011_05630_amd import binding as B
    for (n, hw, c, k), want in (((16, 14, 512, 3), 5), ((16, 56, 256, 3), None), ((16, 28, 512, 3), None)):
        l = B.dlf_i8conv_create(n, hw, hw, c, c, k, True)
        info = B.dlf_i8conv_info(l)
        B.dlf_i8conv_destroy(l)
        assert (info["shape"] == 5) == (want == 5), (n, hw, c, k, info)
    x, wt, sc, b = gen.make_i8_layer(16, 14, 14, 512, 512, 3, seed=9)
    _check("14x14 x 512, the library's choice", x, wt, sc, b, True)
    info = _check("14x14 x 512 + pool, the library's choice", x, wt, sc, b, True, pool=True)
    assert info["shape"] == 5, info


def test_i8_chain_of_four_layers():
    from oracle import oracle
    n, hw, c = 2, 28, 256
    x, _, _, _ = gen.make_i8_layer(n, hw, hw, c, c, 3, seed=7)
    got, ref = x, x
    for i, k in enumerate((3, 1, 3, 3)):
        _, wt, sc, b = gen.make_i8_layer(1, 1, 1, c, c, k, seed=70 + i)
        announce("i8 chain layer", i)
        got, _ = _run(got, wt, sc, b, True)
        ref = oracle.conv2d_i8(ref, wt, sc, b, 1, k // 2, True)
        assert np.array_equal(got, ref), "layer %d" % i
    assert ref.max() > 50


@pytest.mark.parametrize("name", ["vgg_conv3_2", "vgg_conv4_2", "vgg_conv1_2", "res2_reduce", "res4_expand"])
def test_i8conv_benchmarked_layers_sampled_images(name):
    """The layers `bench.py --i8` times, at their full size and in the launch configuration it uses:
    the first, a middle and the last image of the batch against the oracle (images are independent)."""
    import bench
    from oracle import oracle
    _, batch, hw, c, co, k = [l for l in bench.I8_LAYERS if l[0] == name][0]
    x, wt, sc, b = gen.make_i8_layer(batch, hw, hw, c, co, k)
    announce("i8conv", name, x.shape, "cout", co)
    got, info = _run(x, wt, sc, b, True)
    pick = [0, batch // 2 - 1, batch - 1] if hw <= 56 else [batch - 1]
    ref = oracle.conv2d_i8(x[pick], wt, sc, b, 1, k // 2, True)
    assert np.array_equal(got[pick], ref), (name, info)
    assert got.max() == 127 and (got == 0).mean() > 0.2


def test_i8_vgg16_body_equals_oracle_chain():
    """VGG-16's twelve convolutions behind its first layer with their five pools folded in, each layer fed
    the previous one's int8 output, on a 64 x 64 input (maps of 64 .. 4 pixels a side, 2 x 2 after the last
    pool): the chain `bench.py --i8` times at 224 x 224."""
    from oracle import oracle
    x, params = gen.make_i8_chain(2, 64)
    got, ref = x, x
    kinds = []
    for i, (wt, sc, b, pool) in enumerate(params):
        announce("i8 vgg body layer", i, wt.shape, "pool", pool)
        got, info = _run(got, wt, sc, b, True, 0, pool)
        kinds.append(info["shape"])
        ref = oracle.conv2d_i8(ref, wt, sc, b, 1, 1, True)
        if pool:
            ref = oracle.maxpool2x2_i8(ref)
        assert np.array_equal(got, ref), "layer %d" % i
    assert got.shape == (2, 2, 2, 512) and got.max() > 20, (got.shape, int(got.max()))
    assert 5 in kinds and any(k < 5 for k in kinds), kinds         # small-map and block kernels both take part


def test_i8_layers_captured_in_a_hip_graph_replay_to_the_oracle():
    """dlf_i8conv_run only launches a kernel, so a chain of layers (block 3x3, block 1x1, small-map
    kernel) can be captured; every replay, with eager work and synchronisations between the replays,
    must equal the oracle's chain."""
    from oracle import oracle
    from paper_2011_05630_amd import binding as B
    n, hw = 2, 14
    specs = [(3, 128, 512), (1, 512, 512), (3, 512, 64)]
    x, _, _, _ = gen.make_i8_layer(n, hw, hw, 128, 16, 3, seed=91)
    ref, layers, bufs = x, [], [torch.from_numpy(x).cuda()]
    for i, (k, ci, co) in enumerate(specs):
        _, wt, sc, b = gen.make_i8_layer(1, 1, 1, ci, co, k, seed=92 + i)
        ref = oracle.conv2d_i8(ref, wt, sc, b, 1, k // 2, True)
        layers.append(B.dlf_i8conv_create(n, hw, hw, ci, co, k, True, wt, sc, b))
        bufs.append(torch.zeros((n, hw, hw, co), dtype=torch.int8, device="cuda"))
    kinds = [B.dlf_i8conv_info(l)["shape"] for l in layers]
    assert kinds[1] == 5 or kinds[2] == 5, kinds          # the small-map kernel takes part
    try:
        side = torch.cuda.Stream()

        def chain():
            for l, src, dst in zip(layers, bufs[:-1], bufs[1:]):
                B.dlf_i8conv_run(l, src.data_ptr(), dst.data_ptr(), side.cuda_stream)

        with torch.cuda.stream(side):
            chain()                              # first run: one-time kernel set-up, outside the capture
        torch.cuda.synchronize()
        assert np.array_equal(bufs[-1].cpu().numpy(), ref)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            chain()
        torch.cuda.synchronize()
        for _ in range(3):
            for t in bufs[1:]:
                t.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(bufs[-1].cpu().numpy(), ref)
            with torch.cuda.stream(side):
                chain()
            torch.cuda.synchronize()
            assert np.array_equal(bufs[-1].cpu().numpy(), ref)
    finally:
        for l in layers:
            B.dlf_i8conv_destroy(l)
