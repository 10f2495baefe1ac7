"""Pins for the plan-side oracle: operation counts against the numbers the paper prints, the
search-space count against Eq. 4, the enumerator against its closed-form count and tiny brute
force, and Algorithm 1 against hand traces and its invariants."""
import itertools
import math

import pytest

from oracle import plan_oracle as po
from synth import nets
from helpers import paper_values

PV = paper_values()
G = float(2 ** 30)


def total_conv_ops(net):
    shapes = nets.infer_shapes(net)
    tot, nconv = 0, 0
    for L, (_, out) in zip(net["layers"], shapes):
        if L["op"] in ("conv", "dwconv"):
            tot += po.op_count(L, out[0], out[1])
            nconv += 1
    return tot, nconv


def test_eq1_hand_value():
    L = nets.conv(64, 64, 3)
    assert po.op_count(L, 224, 224) == 2 * 224 * 224 * 9 * 64 * 64
    assert po.mac_count(L, 224, 224, batch=3) == 3 * 224 * 224 * 9 * 64 * 64
    assert po.op_count(nets.fc(25088, 4096), 1, 1, batch=16) == 2 * 16 * 25088 * 4096
    assert po.op_count(nets.maxpool(64), 112, 112) == 0
    assert po.mac_count(nets.dwconv(32), 112, 112) == 112 * 112 * 9 * 32


def test_identical_layer_opcounts_printed_in_sec_IVB():
    # printed as 1.72 and 0.43 "GOPs": these are MAC / 2^30 of {512,512,28^2,3^2}, {512,512,14^2,3^2}
    L = nets.conv(512, 512, 3)
    assert round(po.mac_count(L, 28, 28) / G, 2) == PV["conv1_gops"]
    assert round(po.mac_count(L, 14, 14) / G, 2) == PV["conv2_gops"]


def test_equal_opcount_triple_of_sec_IVA():
    a = po.op_count(nets.conv(32, 32, 3), 224, 224)
    b = po.op_count(nets.conv(64, 64, 3), 112, 112)
    c = po.op_count(nets.conv(128, 128, 3), 56, 56)
    assert a == b == c == 2 * 462422016


@pytest.mark.parametrize("name,builder", [("resnet18", nets.resnet18), ("resnet50", nets.resnet50),
                                          ("vgg19", nets.vgg19), ("alexnet", nets.alexnet)])
def test_network_totals_of_table_networks_description(name, builder):
    tot, nconv = total_conv_ops(builder())
    assert nconv == int(PV[name + "_nconv"])
    assert abs(tot / G - PV[name + "_total"]) <= 0.005
    # printed to three significant digits: half a unit of the last printed digit
    tol = 0.005 if name == "vgg19" else 0.0005
    assert abs(tot / G / nconv - PV[name + "_avg"]) <= tol + 1e-9


def test_workload_shapes():
    s = nets.infer_shapes(nets.vgg16())
    assert s[-3][0] == (7, 7, 512) and s[-1][1] == (1, 1, 1000)
    assert len([L for L in nets.vgg16()["layers"] if L["op"] == "conv"]) == 13
    s = nets.infer_shapes(nets.resnet50())
    assert s[0][1] == (112, 112, 64) and s[1][1] == (56, 56, 64)
    assert s[-2][0] == (7, 7, 2048)
    m = nets.mobilenet_v1()
    s = nets.infer_shapes(m)
    assert len([L for L in m["layers"] if L["op"] == "dwconv"]) == 13
    assert s[-2][0] == (7, 7, 1024)
    macs = sum(po.mac_count(L, o[0], o[1]) for L, (_, o) in zip(m["layers"], s))
    assert abs(macs / 1e9 - 0.569) < 0.002
    macs = sum(po.mac_count(L, o[0], o[1]) for L, (_, o) in
               zip(nets.resnet50()["layers"], nets.infer_shapes(nets.resnet50())))
    assert abs(macs / 1e9 - 4.089) < 0.003
    macs = sum(po.mac_count(L, o[0], o[1]) for L, (_, o) in
               zip(nets.vgg16()["layers"], nets.infer_shapes(nets.vgg16())))
    assert abs(macs / 1e9 - 15.47) < 0.01


def test_intensity_eq3():
    assert po.intensity(100, [10, 30, 10]) == 2.0


def test_space_eq4_values():
    # Eq. 4 with 32 MP choices; n = 2 and 3 by hand: 32^2*1 = 1024; 32^2*2 + 32^3*1 = 34816
    assert po.space_eq4(2) == 1024
    assert po.space_eq4(3) == 34816
    s50 = po.space_eq4(50)
    assert s50 == 32 * (33 ** 49 - 1)
    assert abs(s50 / PV["space50"] - 1) < 2e-3
    # adding the single-block term gives the closed form B(1+B)^(n-1)
    for n in (2, 3, 7, 50):
        assert po.space_eq4(n) + 32 == po.count_plans(n, 32)
    assert po.count_plans(2, 32) == 1056 and po.count_plans(3, 32) == 34848


@pytest.mark.parametrize("n,nb", [(1, 4), (2, 4), (3, 2), (4, 3), (6, 4)])
def test_enumerator_count_and_uniqueness(n, nb):
    budgets = tuple(2 ** i for i in range(nb))
    plans = list(po.enumerate_plans(n, budgets))
    assert len(plans) == po.count_plans(n, nb)
    assert len(set(plans)) == len(plans)
    for part, bud in plans:
        assert part[-1] == n - 1 and list(part) == sorted(set(part)) and len(bud) == len(part)


def test_exhaustive_minimum_tiny_hand_case():
    # 3 layers; fusing (0,1) is cheap, everything else expensive; budget 2 halves the cost
    def cost(f, l, b):
        base = {(0, 0): 10, (1, 1): 10, (2, 2): 10, (0, 1): 8, (1, 2): 30, (0, 2): 40}[(f, l)]
        return base * 2 // b
    c, part, bud, visited = po.best_plan_exhaustive(3, (1, 2), cost)
    assert visited == po.count_plans(3, 2)
    assert (c, part, bud) == (8 + 10, (1, 2), (2, 2))


def test_exhaustive_tie_break_order_and_infeasible():
    # all plans cost the same -> fewest groups wins, then lexicographic budgets
    c, part, bud, _ = po.best_plan_exhaustive(3, (4, 2), lambda f, l, b: 0)
    assert (part, bud) == ((2,), (2,))
    # single group infeasible -> two groups, lexicographically smallest group_last
    def cost(f, l, b):
        return None if (f, l) == (0, 2) else 5
    c, part, bud, _ = po.best_plan_exhaustive(3, (1,), cost)
    assert (c, part, bud) == (10, (0, 2), (1, 1))
    assert po.best_plan_exhaustive(2, (1,), lambda f, l, b: None)[0] is None


def _convs(cs):
    return [nets.conv(c, c, 3) for c in cs]


def test_algorithm1_hand_trace_uniform_layers():
    # alpha=1, beta=0, k=1, b=0: MP(layer) = log2(C) = 4 for C=16.  ops 8 each.
    layers = _convs([16, 16, 16, 16])
    ops = [8, 8, 8, 8]
    # crit 3: 8/4=2 <3 ; 16/4=4 >=3 -> close at 1 ; again at 3
    part, mps = po.algorithm1(layers, ops, 3, alpha=1, beta=0, k=1, b=0, allowed=(1, 2, 4, 8))
    assert (part, mps) == ([1, 3], [4, 4])
    # crit 5: 2, 4, 6>=5 -> close at 2; layer 3 left over: 8/4=2 <5 -> tail block
    part, mps = po.algorithm1(layers, ops, 5, alpha=1, beta=0, k=1, b=0, allowed=(1, 2, 4, 8))
    assert (part, mps) == ([2, 3], [4, 4])
    # crit 1: every layer closes its own block
    part, mps = po.algorithm1(layers, ops, 1, alpha=1, beta=0, k=1, b=0, allowed=(1, 2, 4, 8))
    assert (part, mps) == ([0, 1, 2, 3], [4, 4, 4, 4])


def test_algorithm1_hand_trace_mixed_mp_and_rounding():
    # MPs: C=16 -> 4, C=64 -> 6, C=256 -> 8 (alpha=1, beta=0)
    layers = _convs([16, 64, 256, 256])
    ops = [10, 10, 40, 40]
    # crit 4.5: l0: 10/4=2.5 ; l1: avg 5, 20/5=4 ; l2: avg 6, 60/6=10 >= 4.5 -> close at 2,
    # MP = 2^floor(log2 6) = 4 ; l3: avg 8, 40/8 = 5 >= 4.5 -> close at 3 with 8
    part, mps = po.algorithm1(layers, ops, 4.5, alpha=1, beta=0, k=1, b=0,
                              allowed=(1, 2, 4, 8, 16, 32))
    assert (part, mps) == ([2, 3], [4, 8])
    # allowed set without 4: largest allowed value not above 4 is 2; 8 stays 8
    part, mps = po.algorithm1(layers, ops, 4.5, alpha=1, beta=0, k=1, b=0, allowed=(2, 8, 32))
    assert (part, mps) == ([2, 3], [2, 8])


def test_algorithm1_pool_layers_ride_with_preceding_block():
    layers = [nets.maxpool(16), nets.conv(16, 16, 3), nets.maxpool(16), nets.conv(16, 16, 3),
              nets.maxpool(16), nets.gavgpool(16)]
    ops = [0, 8, 0, 8, 0, 0]
    # a leading pool opens the block without dividing by zero; crit 2 closes after each conv and
    # the pools that follow ride along
    part, mps = po.algorithm1(layers, ops, 2, alpha=1, beta=0, k=1, b=0, allowed=(1, 2, 4))
    assert (part, mps) == ([2, 5], [4, 4])
    # never reaching the threshold: one block holding everything
    part, mps = po.algorithm1(layers, ops, 1000, alpha=1, beta=0, k=1, b=0, allowed=(1, 2, 4))
    assert (part, mps) == ([5], [4])


def test_layer_mp_eq5_form():
    L = nets.conv(64, 128, 3)
    ops = 2 ** 30
    # alpha*log2(min(Cin,Cout)) + beta*log2(ops) with the paper's constants
    exp = 0.316 * 6 + 0.659 * 30
    assert po.layer_mp(L, ops, 0.316, 0.659, 1.0, 0.0, 32) == pytest.approx(exp)
    assert po.layer_mp(L, ops, 0.316, 0.659, 1.0, 0.0, 16) == 16.0      # clamp high
    assert po.layer_mp(L, ops, 0.316, 0.659, 0.0, -5.0, 32) == 1.0      # clamp low
    # monotone in both features
    assert po.layer_mp(nets.conv(128, 128, 3), ops, 0.316, 0.659, 1, 0, 64) > \
        po.layer_mp(nets.conv(64, 64, 3), ops, 0.316, 0.659, 1, 0, 64)
    assert po.layer_mp(L, 2 * ops, 0.316, 0.659, 1, 0, 64) > po.layer_mp(L, ops, 0.316, 0.659, 1,
                                                                        0, 64)


@pytest.mark.parametrize("builder", [nets.vgg16, nets.resnet50, nets.mobilenet_v1, nets.alexnet])
def test_algorithm1_invariants_on_real_shapes(builder):
    net = builder()
    shapes = nets.infer_shapes(net)
    ops = [po.op_count(L, o[0], o[1]) for L, (_, o) in zip(net["layers"], shapes)]
    allowed = (1, 2, 4, 8, 16, 32)
    for crit in (1e6, 1e8, 10 ** 1.25 * G, 1e12):
        part, mps = po.algorithm1(net["layers"], ops, crit, k=1.0, b=-8.0, allowed=allowed)
        n = len(ops)
        assert part[-1] == n - 1 and part == sorted(set(part)) and len(part) == len(mps)
        assert all(m in allowed for m in mps)
        first = 0
        for gi, last in enumerate(part):
            blk = range(first, last + 1)
            assert net["layers"][first]["op"] in po.CONV_LIKE or first == 0
            convs = [i for i in blk if net["layers"][i]["op"] in po.CONV_LIKE]
            if gi < len(part) - 1:
                mp = [po.layer_mp(net["layers"][i], ops[i], 0.316, 0.659, 1.0, -8.0, 32)
                      for i in convs]
                avg = sum(mp) / len(mp)
                assert sum(ops[i] for i in convs) / avg >= crit
                # greedy: dropping the last conv layer of the block leaves it below the threshold
                if len(convs) > 1:
                    avg2 = sum(mp[:-1]) / (len(mp) - 1)
                    assert sum(ops[i] for i in convs[:-1]) / avg2 < crit
            first = last + 1


def test_layerwise_budgets_hand_trace():
    """The no-fusion rows of the table of strategies (Sec. V): strategy 3 gives every layer the MP of
    Eq. 5 rounded as a one-layer block; strategies 1 and 2 give every layer one fixed MP.  With
    alpha = 1, beta = 0, k = 1, b = 0 the per-layer MP is log2(min(Cin, Cout))."""
    layers = [nets.maxpool(16), nets.conv(16, 64, 3), nets.maxpool(64), nets.conv(64, 256, 1),
              nets.conv(256, 48, 3), nets.gavgpool(48), nets.fc(48, 1000)]
    ops = [0, 100, 0, 100, 100, 0, 100]
    # log2 C: conv0 min(16,64) -> 4 ; conv1 min(64,256) -> 6 -> 2^2 = 4 ; conv2 min(256,48) -> 5.58 -> 4
    # fc min(48,1000) -> 5.58 -> 4.  A leading pool has no convolution before it: smallest allowed MP;
    # later pools take the MP of the convolution before them.
    got = po.layerwise_budgets(layers, ops, alpha=1, beta=0, k=1, b=0, allowed=(1, 2, 4, 8))
    assert got == [1, 4, 4, 4, 4, 4, 4]
    # k = 2: MPs 8, 12 -> 8, 11.17 -> 8, 11.17 -> 8 clamped to max 8
    got = po.layerwise_budgets(layers, ops, alpha=1, beta=0, k=2, b=0, allowed=(1, 2, 4, 8))
    assert got == [1, 8, 8, 8, 8, 8, 8]
    # an allowed set without 4: 2^floor(log2 x) = 4 falls to the largest allowed value below, 2;
    # beta = 1 on ops 2^3 / 2^5: MP = log2 ops -> 3 -> 2 ; 5 -> 4 -> 2 ... ; ops 2^7 -> 7 -> 4 -> 2 ; 2^9 -> 9 -> 8
    layers2 = [nets.conv(16, 16, 3), nets.maxpool(16), nets.conv(16, 16, 3), nets.conv(16, 16, 3)]
    got = po.layerwise_budgets(layers2, [2 ** 3, 0, 2 ** 7, 2 ** 9], alpha=0, beta=1, k=1, b=0,
                               allowed=(2, 8, 32))
    assert got == [2, 2, 2, 8]
    # one MP for all (strategies 1 and 2), pools included
    assert po.layerwise_budgets(layers, ops, fixed_budget=16) == [16] * 7


def test_max_fusion_hand_trace():
    """Strategy 4 of the table of strategies (everything fused, maximal MP), as far as a
    feasibility test lets blocks grow: the longest feasible block from the left, again and again."""
    # feasible iff the block has at most 3 layers
    assert po.max_fusion(7, lambda f, l: l - f < 3, 32) == [(0, 2, 32), (3, 5, 32), (6, 6, 32)]
    # everything feasible: one block
    assert po.max_fusion(5, lambda f, l: True, 8) == [(0, 4, 8)]
    # only single layers feasible
    assert po.max_fusion(3, lambda f, l: f == l, 4) == [(0, 0, 4), (1, 1, 4), (2, 2, 4)]
    # a feasibility test that is not monotone: [0,3] is infeasible, [0,2] too, [0,1] feasible;
    # then [2,4] feasible
    ok = {(0, 1), (2, 4), (0, 0), (1, 1), (2, 2), (3, 3), (4, 4), (2, 3)}
    assert po.max_fusion(5, lambda f, l: (f, l) in ok, 2) == [(0, 1, 2), (2, 4, 2)]
    # a layer that cannot run even alone is the caller's error
    with pytest.raises(AssertionError):
        po.max_fusion(2, lambda f, l: False, 2)
