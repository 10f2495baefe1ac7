"""Host-side checks that need no GPU: the library loads and exports its whole C ABI, its exact
tuner returns the plan that brute-force enumeration finds over the library's own published cost
table (Sec. V, "Oracle Case", on nets small enough to enumerate), its greedy mode follows
Algorithm 1, and bad arguments are rejected with an error."""
import os
import random
import re

import pytest

from synth import nets
from oracle import plan_oracle as P
from paper_2011_05630_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BUDGETS = (32, 64, 128, 256)


def _net(layers, h, w, c, name="t"):
    return dict(name=name, layers=layers, in_h=h, in_w=w, in_c=c, input_dist="uniform")


def _handle(net):
    return B.dlf_net_create(net["layers"], net["in_h"], net["in_w"], net["in_c"])


def _sub(net, first, last):
    """Layers [first, last] of a net as a net of their own (chains only)."""
    h, w, c = nets.infer_shapes(net)[first][0]
    layers = []
    for i in range(first, last + 1):
        L = dict(net["layers"][i])
        for key in ("input_from", "residual_from"):
            if L[key] >= 0:
                L[key] -= first
                assert L[key] >= 0 or key == "input_from" and L[key] == -1
        layers.append(L)
    return _net(layers, h, w, c, "%s[%d:%d]" % (net["name"], first, last))


def _random_net(rng):
    """A legal random layer list: convolutions, depthwise, pooling, strides, one residual."""
    c = rng.choice([8, 16, 32, 64])
    hw = rng.choice([14, 20, 28, 33])
    layers, shapes = [], []
    h = w = hw
    cin = c
    n = rng.randint(3, 7)
    for i in range(n):
        kind = rng.choice(["c3", "c3", "c1", "dw", "pool", "c3s2"])
        if kind == "pool" and (min(h, w) < 4 or i == 0):
            kind = "c3"
        if kind == "c3s2" and min(h, w) < 6:
            kind = "c3"
        if kind == "c3":
            cout = rng.choice([16, 32, 64])
            layers.append(nets.conv(cin, cout, 3, 1, 1, "relu"))
        elif kind == "c3s2":
            cout = rng.choice([32, 64])
            layers.append(nets.conv(cin, cout, 3, 2, 1, "relu"))
            h, w = (h - 1) // 2 + 1, (w - 1) // 2 + 1
        elif kind == "c1":
            cout = rng.choice([16, 32, 64, 128])
            layers.append(nets.conv(cin, cout, 1, 1, 0, "relu6"))
        elif kind == "dw":
            cout = cin
            layers.append(nets.dwconv(cin, 3, 1, "relu6"))
        else:
            cout = cin
            k = rng.choice([2, 3])
            layers.append(nets.maxpool(cin, k, 2, 0 if k == 2 else 1))
            h, w = ((h - 2) // 2 + 1, (w - 2) // 2 + 1) if k == 2 else ((h - 1) // 2 + 1, (w - 1) // 2 + 1)
        cin = cout
        shapes.append((h, w, cout))
    # a residual add onto the last layer from an earlier tensor of the same shape, if any
    if layers[-1]["op"] == "conv":
        same = [j for j in range(n - 1) if shapes[j] == shapes[-1]]
        if same and rng.random() < 0.6:
            layers[-1]["residual_from"] = rng.choice(same)
    return _net(layers, hw, hw, c, "rand")


def _small_nets():
    out = [(nets.two_layer_block(), 1)]
    for c in (16, 64, 256):
        out.append((nets.chain4(c), 1))
        out.append((nets.chain4(c), 8))
    v = nets.vgg16()
    out.append((_sub(v, 0, 6), 16))        # conv conv pool conv conv pool conv
    out.append((_sub(v, 10, 17), 1))       # deep 512-channel stages with pools
    r = nets.resnet50()
    out.append((_sub(r, 0, 5), 32))        # stem, pool, first bottleneck with projection
    out.append((_sub(r, 0, 8), 4))         # ... plus an identity bottleneck
    m = nets.mobilenet_v1()
    out.append((_sub(m, 0, 6), 64))        # stem + three dw/pw pairs
    out.append((_sub(m, len(m["layers"]) - 6, len(m["layers"]) - 1), 64))   # ... gap, fc
    out.append((nets.alexnet(), 4))
    rng = random.Random(5630)
    for _ in range(8):
        out.append((_random_net(rng), rng.choice([1, 2, 8])))
    return out


SMALL = _small_nets()


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "dlf.h")).read() + open(os.path.join(ROOT, "include", "dlf_debug.h")).read()
    assert "dlf_debug_" not in open(os.path.join(ROOT, "include", "dlf.h")).read()     # hooks live in their own header
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    hdr = re.sub(r"//[^\n]*", "", hdr)
    names = sorted(set(re.findall(r"\b(dlf_[a-z0-9_]+)\s*\(", hdr)))
    assert len(names) >= 20, names
    lib = B.lib()
    missing = [n for n in names if not hasattr(lib, n)]
    assert not missing, missing
    # and the binding offers the same names
    unbound = [n for n in names if not hasattr(B, n)]
    assert not unbound, unbound
    assert B.dlf_cost_model_version() == 3


def test_layer_info_matches_eq1_eq2():
    for net in (nets.vgg16(), nets.resnet50(), nets.mobilenet_v1()):
        h = _handle(net)
        shapes = nets.infer_shapes(net)
        for i, L in enumerate(net["layers"]):
            oh, ow, oc, ops = B.dlf_net_layer_info(h, i)
            assert (oh, ow, oc) == tuple(shapes[i][1])
            assert ops == P.op_count(L, oh, ow)
        B.dlf_net_destroy(h)


def _cost_table(h, batch, n, budgets, lds=0):
    """The library's published cost function, read range by range (None = cannot run as a group)."""
    return {(f, l, b): B.dlf_group_cost(h, batch, f, l, b, lds)
            for f in range(n) for l in range(f, n) for b in budgets}


@pytest.mark.parametrize("idx", range(len(SMALL)))
def test_group_cost_table_is_well_formed(idx):
    """What an exhaustive search over the table relies on: every single layer can run alone, a
    range that holds an FC or global pooling layer together with anything else cannot, the values
    do not depend on the order of the calls, and no group is modelled below a microsecond (every
    group pays for its launch)."""
    net, batch = SMALL[idx]
    h = _handle(net)
    n = len(net["layers"])
    t1 = _cost_table(h, batch, n, (1, 7) + BUDGETS)
    t2 = _cost_table(h, batch, n, (1, 7) + BUDGETS)
    assert t1 == t2
    for i in range(n):
        for b in BUDGETS:
            assert t1[(i, i, b)] is not None and t1[(i, i, b)] > 0
    for (f, l, b), c in t1.items():
        ops = [net["layers"][i]["op"] for i in range(f, l + 1)]
        if l > f and any(o in ("fc", "gavgpool") for o in ops):
            assert c is None, (f, l, ops)
        if c is not None:
            assert c >= 1000 * 1000          # no group is modelled below a microsecond
    B.dlf_net_destroy(h)


def test_group_cost_respects_lds_limit():
    """A larger on-chip memory limit only adds candidate tilings: the minimum never rises, and a
    4-deep 64-channel chain that fits 160 KiB does not fit 16 KiB."""
    net = nets.chain4(64)
    h = _handle(net)
    seen = set()
    limits = (16 * 1024, 40 * 1024, 64 * 1024, 160 * 1024)
    for l in range(4):
        prev = None
        for lds in limits:
            got = B.dlf_group_cost(h, 1, 0, l, 256, lds)
            seen.add((lds, l, got is not None))
            if prev is not None:
                assert got is not None and got <= prev
            prev = got if got is not None else prev
    assert (16 * 1024, 3, False) in seen and (160 * 1024, 3, True) in seen
    B.dlf_net_destroy(h)


def _plan_tuple(h, batch, **kw):
    p = B.dlf_plan(h, batch, **kw)
    gs = B.dlf_plan_groups(p)
    B.dlf_plan_destroy(p)
    return (sum(g["model_cost"] for g in gs), tuple(g["last"] for g in gs),
            tuple(g["budget"] for g in gs)), gs


@pytest.mark.parametrize("idx", range(len(SMALL)))
def test_dp_plan_equals_exhaustive_search(idx):
    net, batch = SMALL[idx]
    n = len(net["layers"])
    budgets = BUDGETS if n <= 7 else (64, 256)
    assert P.count_plans(n, len(budgets)) <= 400000
    h = _handle(net)
    table = _cost_table(h, batch, n, budgets)
    cost, lasts, buds, visited = P.best_plan_exhaustive(n, budgets, lambda f, l, b: table[(f, l, b)])
    assert visited == P.count_plans(n, len(budgets))
    got, gs = _plan_tuple(h, batch, mode=B.TUNER_DP, budgets=list(budgets))
    assert got == (cost, lasts, buds), (net["name"], got, (cost, lasts, buds))
    # groups tile the layer list
    first = 0
    for g in gs:
        assert g["first"] == first
        first = g["last"] + 1
    assert first == n
    B.dlf_net_destroy(h)


@pytest.mark.parametrize("name,batch", [("vgg16", 16), ("resnet50", 32), ("mobilenet_v1", 64),
                                        ("resnet18", 8), ("alexnet", 4)])
def test_dp_plan_is_no_worse_than_any_other_mode_on_full_networks(name, batch):
    """Where enumeration is out of reach the optimum still bounds every plan the other modes
    build from the same cost table: its total modelled cost is not above theirs, and it equals
    the sum of the table entries of its own groups."""
    net = getattr(nets, name)()
    h = _handle(net)
    (dp_cost, lasts, buds), gs = _plan_tuple(h, batch)
    assert dp_cost == sum(B.dlf_group_cost(h, batch, g["first"], g["last"], g["budget"]) for g in gs)
    n = len(net["layers"])
    others = [dict(mode=B.TUNER_GREEDY), dict(mode=B.TUNER_LAYERWISE), dict(mode=B.TUNER_MAXFUSE),
              dict(mode=B.TUNER_MANUAL, group_last=list(range(n)), group_budget=[256] * n),
              dict(mode=B.TUNER_MANUAL, group_last=list(range(n)), group_budget=[64] * n)]
    for kw in others:
        (c, _, _), _ = _plan_tuple(h, batch, **kw)
        assert dp_cost <= c, (kw, dp_cost, c)
    B.dlf_net_destroy(h)


def test_dp_plan_under_a_small_lds_limit():
    net = nets.chain4(32)
    h = _handle(net)
    for lds in (24 * 1024, 64 * 1024):
        table = _cost_table(h, 2, 4, BUDGETS, lds)
        cost, lasts, buds, _ = P.best_plan_exhaustive(4, BUDGETS, lambda f, l, b: table[(f, l, b)])
        got, _ = _plan_tuple(h, 2, mode=B.TUNER_DP, budgets=list(BUDGETS), max_lds_bytes=lds)
        assert got == (cost, lasts, buds)
    B.dlf_net_destroy(h)


def test_dp_fuses_where_the_model_says_so():
    """Sanity of the plan itself: small feature maps fuse, and the fused plan's modelled cost is
    below the all-separate plan's."""
    net = nets.two_layer_block()
    h = _handle(net)
    (cost, lasts, buds), _ = _plan_tuple(h, 1)
    sep = sum(B.dlf_group_cost(h, 1, i, i, 256) for i in range(2))
    assert lasts == (1,) and cost < sep
    B.dlf_net_destroy(h)


def _legalise(h, batch, part, mps):
    """Blocks of Algorithm 1 -> executable groups: each block is cut left to right into the
    longest groups the kernels can run (the library's own feasibility answer), all with the
    block's MP."""
    out = []
    first = 0
    for blk_last, mp in zip(part, mps):
        while first <= blk_last:
            l = blk_last
            while B.dlf_group_cost(h, batch, first, l, mp) is None:
                l -= 1
                assert l >= first
            out.append((first, l, mp))
            first = l + 1
    return out


@pytest.mark.parametrize("name,batch", [("two_layer_block", 1), ("vgg16", 1), ("vgg16", 16),
                                        ("resnet50", 32), ("mobilenet_v1", 64), ("alexnet", 4),
                                        ("resnet18", 8)])
@pytest.mark.parametrize("crit,k,b", [(2.0e7, 16.0, -256.0), (5.0e8, 8.0, -100.0), (1.0e6, 1.0, 0.0)])
def test_greedy_mode_follows_algorithm1(name, batch, crit, k, b):
    net = getattr(nets, name)()
    osh = [o for _, o in nets.infer_shapes(net)]
    ops = [P.op_count(L, osh[i][0], osh[i][1], batch) for i, L in enumerate(net["layers"])]
    part, mps = P.algorithm1(net["layers"], ops, crit, 0.316, 0.659, k, b, BUDGETS)
    assert part[-1] == len(net["layers"]) - 1 and len(part) == len(mps)
    h = _handle(net)
    want = _legalise(h, batch, part, mps)
    p = B.dlf_plan(h, batch, mode=B.TUNER_GREEDY, budgets=list(BUDGETS), opcount_critical=crit,
                   alpha=0.316, beta=0.659, mp_scale=k, mp_offset=b)
    got = [(g["first"], g["last"], g["budget"]) for g in B.dlf_plan_groups(p)]
    B.dlf_plan_destroy(p)
    B.dlf_net_destroy(h)
    assert got == want


@pytest.mark.parametrize("name,batch", [("vgg16", 16), ("resnet50", 32), ("mobilenet_v1", 64),
                                        ("alexnet", 4), ("two_layer_block", 1)])
def test_comparison_strategies_of_the_evaluation(name, batch):
    """The other rows of the paper's table of strategies: no fusion with one MP for all layers
    (1, 2), no fusion with Eq. 5 per layer (3), maximal fusion on the largest MP (4), Algorithm 1
    with one MP for all blocks (5)."""
    net = getattr(nets, name)()
    n = len(net["layers"])
    osh = [o for _, o in nets.infer_shapes(net)]
    ops = [P.op_count(L, osh[i][0], osh[i][1], batch) for i, L in enumerate(net["layers"])]
    h = _handle(net)

    def groups(**kw):
        p = B.dlf_plan(h, batch, budgets=list(BUDGETS), **kw)
        g = [(g["first"], g["last"], g["budget"]) for g in B.dlf_plan_groups(p)]
        B.dlf_plan_destroy(p)
        return g

    k, b, crit = 16.0, -256.0, 2.0e7
    want = P.layerwise_budgets(net["layers"], ops, 0.316, 0.659, k, b, BUDGETS)
    assert groups(mode=B.TUNER_LAYERWISE, mp_scale=k, mp_offset=b) == [(i, i, want[i]) for i in range(n)]
    assert groups(mode=B.TUNER_LAYERWISE, fixed_budget=64) == [(i, i, 64) for i in range(n)]
    feasible = lambda f, l: B.dlf_group_cost(h, batch, f, l, max(BUDGETS)) is not None
    assert groups(mode=B.TUNER_MAXFUSE) == P.max_fusion(n, feasible, max(BUDGETS))
    part, mps = P.algorithm1(net["layers"], ops, crit, 0.316, 0.659, k, b, BUDGETS)
    assert groups(mode=B.TUNER_GREEDY, opcount_critical=crit, mp_scale=k, mp_offset=b, fixed_budget=128) == \
        _legalise(h, batch, part, [128] * len(part))
    B.dlf_net_destroy(h)


def test_greedy_defaults_are_the_documented_ones():
    net = nets.resnet50()
    h = _handle(net)
    p = B.dlf_plan(h, 32, mode=B.TUNER_GREEDY)
    a = [(g["first"], g["last"], g["budget"]) for g in B.dlf_plan_groups(p)]
    B.dlf_plan_destroy(p)
    p = B.dlf_plan(h, 32, mode=B.TUNER_GREEDY, budgets=list(BUDGETS), opcount_critical=2.0e7,
                   alpha=0.316, beta=0.659, mp_scale=64.0, mp_offset=-1056.0)
    b = [(g["first"], g["last"], g["budget"]) for g in B.dlf_plan_groups(p)]
    B.dlf_plan_destroy(p)
    B.dlf_net_destroy(h)
    assert a == b


def test_manual_plan_and_workspace():
    net = nets.chain4(64)
    h = _handle(net)
    p = B.dlf_plan(h, 8, mode=B.TUNER_MANUAL, group_last=[1, 3], group_budget=[64, 256])
    gs = B.dlf_plan_groups(p)
    assert [(g["first"], g["last"], g["budget"]) for g in gs] == [(0, 1, 64), (2, 3, 256)]
    assert gs[0]["model_cost"] == B.dlf_group_cost(h, 8, 0, 1, 64)
    # one intermediate tensor (layer 1's output), 256-byte aligned
    assert B.dlf_plan_workspace_bytes(p) == 8 * 56 * 56 * 64 * 2
    assert B.dlf_plan_group_io(p, 0) == (-1, -2) and B.dlf_plan_group_io(p, 1) == (1, -2)
    B.dlf_plan_destroy(p)
    B.dlf_net_destroy(h)


def test_residual_groups_read_their_operand_from_outside():
    r = nets.resnet50()
    net = _sub(r, 0, 5)              # stem, pool, 1x1, 3x3, projection, 1x1 + projection result
    h = _handle(net)
    # the projection shortcut and the block's last layer as one group of two 1x1 convolutions that
    # reads both their inputs (the planner's choice here) ...
    p = B.dlf_plan(h, 2)
    gs = B.dlf_plan_groups(p)
    last = len(gs) - 1
    assert (gs[last]["first"], gs[last]["last"]) == (4, 5)
    assert B.dlf_plan_group_config(p, last)["kind"] == 8
    assert B.dlf_plan_group_io(p, last) == (3, 1)       # the 3x3 layer's output, the block input
    B.dlf_plan_destroy(p)
    # ... and, with the pointwise kernels switched off, the last layer adding the projection's
    # result from memory: a residual operand is never produced inside the group that adds it
    B.dlf_debug_pointwise_mode(2)
    try:
        p = B.dlf_plan(h, 2)
    finally:
        B.dlf_debug_pointwise_mode(0)
    gs = B.dlf_plan_groups(p)
    last = len(gs) - 1
    assert gs[last]["last"] == 5
    in_layer, res_layer = B.dlf_plan_group_io(p, last)
    assert res_layer == net["layers"][5]["residual_from"]
    assert not (gs[last]["first"] <= res_layer <= gs[last]["last"])
    B.dlf_plan_destroy(p)
    B.dlf_net_destroy(h)


def _raises(status_substr, fn, *a, **kw):
    with pytest.raises(B.DlfError) as e:
        fn(*a, **kw)
    assert status_substr in str(e.value).lower(), str(e.value)


def test_error_paths_on_the_host():
    good = nets.chain4(16)
    h = _handle(good)
    _raises("manual", B.dlf_plan, h, 1, mode=B.TUNER_MANUAL, group_last=[1], group_budget=[64])
    _raises("manual", B.dlf_plan, h, 1, mode=B.TUNER_MANUAL, group_last=[2, 1, 3], group_budget=[64] * 3)
    _raises("budget", B.dlf_plan, h, 1, budgets=[0, 64])
    _raises("mode", B.dlf_plan, h, 1, mode=7)
    _raises("argument", B.dlf_plan, h, 0)
    _raises("group", B.dlf_plan, h, 1, mode=B.TUNER_MANUAL, group_last=[3], group_budget=[0])
    assert B.dlf_group_cost(h, 1, 0, 3, 64, 8 * 1024) is None       # nothing fits 8 KiB
    B.dlf_net_destroy(h)
    bad = [dict(nets.conv(16, 16)), dict(nets.conv(32, 16))]        # cin mismatch
    _raises("cin", B.dlf_net_create, bad, 8, 8, 16)
    bad = [dict(nets.conv(16, 18))]                                   # cout % 4
    _raises("cout", B.dlf_net_create, bad, 8, 8, 16)
    bad = [dict(nets.conv(16, 16)), dict(nets.conv(16, 16, residual_from=1))]
    _raises("earlier", B.dlf_net_create, bad, 8, 8, 16)
    bad = [dict(nets.conv(16, 32)), dict(nets.conv(32, 16, residual_from=0))]
    _raises("residual", B.dlf_net_create, bad, 8, 8, 16)
    bad = [dict(nets.conv(16, 16, 5, 1, 0))]
    _raises("kernel", B.dlf_net_create, bad, 3, 3, 16)
    _raises("non-positive", B.dlf_net_create, [dict(nets.conv(16, 16))], 0, 8, 16)
    # a net without weights plans but does not run
    h = _handle(good)
    p = B.dlf_plan(h, 1)
    _raises("weight", B.dlf_run, p, 256, 256)
    B.dlf_plan_destroy(p)
    B.dlf_net_destroy(h)


def test_i8conv_shape_only_layer_and_argument_checks():
    """The quantised layer's host side without a GPU: a shape-only layer reports its tile, refuses
    to run, and unsupported or invalid sizes come back as statuses."""
    l = B.dlf_i8conv_create(16, 56, 56, 256, 256, 3, True)
    info = B.dlf_i8conv_info(l)
    assert info["op_count"] == 2 * 16 * 56 * 56 * 9 * 256 * 256        # Eq. 1 over the batch
    assert info["th"] * info["tw"] <= 512 and info["grid"] % 8 == 0 and 8 <= info["grid"] <= 256
    with pytest.raises(B.DlfError) as e:
        B.dlf_i8conv_run(l, 16, 16, None)
    assert e.value.status == B.DLF_ERR_NO_WEIGHTS
    B.dlf_i8conv_destroy(l)
    l = B.dlf_i8conv_create(32, 28, 28, 512, 128, 1, False)
    info = B.dlf_i8conv_info(l)
    assert info["op_count"] == 2 * 32 * 28 * 28 * 512 * 128 and info["th"] == 1 and info["tw"] in (128, 256)
    B.dlf_i8conv_destroy(l)
    with pytest.raises(B.DlfError) as e:
        B.dlf_i8conv_create(1, 8, 8, 64, 64, 5, False)
    assert e.value.status == B.DLF_ERR_UNSUPPORTED
    for bad, st in (((1, 8, 8, 48, 64), B.DLF_ERR_UNSUPPORTED), ((1, 8, 8, 64, 24), B.DLF_ERR_UNSUPPORTED),
                    ((0, 8, 8, 64, 64), B.DLF_ERR_INVALID_ARG), ((1, 8, 8, 64, -16), B.DLF_ERR_INVALID_ARG),
                    ((64, 1024, 1024, 64, 64), B.DLF_ERR_UNSUPPORTED)):
        with pytest.raises(B.DlfError) as e:
            B.dlf_i8conv_create(*bad, 3, False)
        assert e.value.status == st, bad
