"""GPU parity of the five synthetic workloads against the CPU oracle, through the C ABI.

Small batches are compared element by element on the whole output.  At the large batch of a
workload the oracle is run on sampled images only (images are independent, so each sampled
image's output is computed exactly as in a full run), in the same launch configuration the
benchmark times.  Every fusion group of the tuned plan is also checked on its own, the oracle
being fed the GPU's own group input, so errors cannot hide behind later layers."""
import numpy as np
import pytest
import torch

from synth import nets, gen
from gpu_util import compare, announce

pytestmark = pytest.mark.gpu


def _session(net, batch, ws, bs, **plan):
    from paper_2011_05630_amd.runner import Session
    return Session(net, batch, ws, bs, **plan)


def _manual(lasts, budget):
    from paper_2011_05630_amd import binding as B
    return dict(mode=B.TUNER_MANUAL, group_last=list(lasts), group_budget=[budget] * len(lasts))


KIND_NAME = {0: "group", 1: "fc", 2: "gap", 3: "pw", 4: "c3b", 5: "dw", 6: "dwpw", 7: "dwt", 8: "pw2", 9: "dws", 10: "c3s", 11: "c3pw", 12: "bneck"}


def _kinds(s):
    """(kind name, variant) of every group of the session's plan, as the library reports them."""
    from paper_2011_05630_amd import binding as B
    out = []
    for g in range(len(s.groups)):
        cfg = B.dlf_plan_group_config(s.plan, g)
        out.append((KIND_NAME[cfg["kind"]], cfg["variant"]))
    return out


def _check_groups(s, net, x, ws, bs, sample=None):
    """Each group's output vs the oracle applied to the GPU's own input of that group, on the
    images `sample` of the batch (all images if None): images are independent, so a sampled
    image's tensors are exactly those of a full run."""
    from oracle import oracle as o
    n = len(net["layers"])
    idx = list(range(x.shape[0])) if sample is None else list(sample)
    tidx = torch.tensor(idx, device="cuda")
    outs = {-1: x[idx].astype(np.float32)}
    for i in range(n):
        t = s.layer_output(i)
        if t is not None:
            outs[i] = t.index_select(0, tidx).float().cpu().numpy()
    checked = 0
    for g in s.groups:
        if g["last"] == n - 1:
            continue
        given = {k: v for k, v in outs.items() if k < g["first"]}
        ref = o.run_net(net, None, ws, bs, first=g["first"], last=g["last"], given=given)
        compare(outs[g["last"]], ref, "  group [%d,%d]" % (g["first"], g["last"]))
        checked += 1
    assert checked == len(s.groups) - 1


def test_config1_two_layer_block_fused_vs_unfused():
    from oracle import oracle as o
    net = nets.two_layer_block()
    x, ws, bs = gen.make_params(net, 1)
    ref = o.run_net(net, x, ws, bs)
    res = {}
    for name, lasts in (("fused", [1]), ("unfused", [0, 1])):
        for budget in (32, 64, 128, 256):
            announce("config1", name, budget)
            s = _session(net, 1, ws, bs, **_manual(lasts, budget))
            got = s.run_numpy(x)
            s.close()
            compare(got, ref, "config1 %s budget %d" % (name, budget))
            res[(name, budget)] = got
    # the budget never changes the arithmetic
    for name in ("fused", "unfused"):
        for budget in (64, 128, 256):
            assert np.array_equal(res[(name, budget)], res[(name, 32)])


PARTITIONS = {1: [0, 1, 2, 3], 2: [1, 3], 3: [2, 3], 4: [3]}


@pytest.mark.parametrize("c", [16, 32, 64, 128, 256])
@pytest.mark.parametrize("batch", [1, 8])
def test_config2_layer_sweep(c, batch):
    from oracle import oracle as o
    net = nets.chain4(c)
    x, ws, bs = gen.make_params(net, batch)
    ref = o.run_net(net, x, ws, bs)
    ran = 0
    # every one of the 16 (depth, budget) points of every width fits on-chip memory (with smaller
    # tiles as the width grows): a point that stops fitting raises here
    for depth, lasts in PARTITIONS.items():
        for budget in (32, 64, 128, 256):
            announce("config2 C", c, "batch", batch, "depth", depth, "budget", budget)
            s = _session(net, batch, ws, bs, **_manual(lasts, budget))
            assert [g["last"] for g in s.groups] == lasts
            got = s.run_numpy(x)
            s.close()
            compare(got, ref, "config2 C=%d b=%d depth=%d budget=%d" % (c, batch, depth, budget))
            ran += 1
    assert ran == 16


def _net_case(net, batch, sample, check_groups, plans, expect_kinds=()):
    """expect_kinds: (kind name, variant or None) pairs the first plan must contain: the kernels the
    cost model is known to pick for this workload, so that a silent change of the planner's choice
    (and with it of what this test covers) shows."""
    from oracle import oracle as o
    x, ws, bs = gen.make_params(net, batch)
    xs = x[sample]
    ref = o.run_net(net, xs, ws, bs)
    for pi, (pname, plan) in enumerate(plans):
        announce(net["name"], "batch", batch, "plan", pname)
        s = _session(net, batch, ws, bs, **plan)
        kinds = _kinds(s)
        print("  groups:", [(g["first"], g["last"], g["budget"]) + k for g, k in zip(s.groups, kinds)])
        if pi == 0:
            for kind, variant in expect_kinds:
                assert any(k == kind and (variant is None or v == variant) for k, v in kinds), \
                    "plan holds no %s%s group: %r" % (kind, "" if variant is None else "/%d" % variant, kinds)
        got = s.run_numpy(x)
        compare(got[sample], ref, "%s b=%d %s" % (net["name"], batch, pname))
        if check_groups:
            _check_groups(s, net, x, ws, bs, sample)
        s.close()


def _plans(net):
    from paper_2011_05630_amd import binding as B
    n = len(net["layers"])
    return [("dp", dict(mode=B.TUNER_DP)), ("greedy", dict(mode=B.TUNER_GREEDY)),
            ("unfused", _manual(list(range(n)), 256))]


def test_config3_vgg16_batch1():
    net = nets.vgg16()
    _net_case(net, 1, [0], True, _plans(net))


def test_config3_vgg16_batch16_sampled():
    net = nets.vgg16()
    # the plan the benchmark times: block 3x3 kernel on the wide layers, split-K FC on 25088 -> 4096
    _net_case(net, 16, [0, 7, 15], True, _plans(net)[:1], expect_kinds=[("c3b", None), ("c3s", None), ("group", None), ("fc", None)])


def test_config4_resnet50_batch1():
    net = nets.resnet50()
    _net_case(net, 1, [0], True, _plans(net))


def test_config4_resnet50_batch32_sampled():
    net = nets.resnet50()
    # image 17: its pixels straddle the 128-pixel blocks of the pointwise block kernel on every map;
    # the small-map kernel on the 3x3 (variant = waves per channel block) and 1x1 (8 + that) layers of the last two stages
    _net_case(net, 32, [0, 17, 31], True, _plans(net)[:1],
              expect_kinds=[("pw", 3), ("pw2", None), ("group", None), ("c3s", 2), ("c3s", 10), ("c3pw", 4), ("bneck", 256)])


def test_config5_mobilenet_batch1():
    net = nets.mobilenet_v1()
    _net_case(net, 1, [0], True, _plans(net))


def test_config5_mobilenet_batch64_sampled():
    net = nets.mobilenet_v1()
    _net_case(net, 64, [0, 33, 63], True, _plans(net)[:1], expect_kinds=[("pw", None), ("dw", 0), ("dw", 1), ("dwt", 0), ("dwt", 1), ("dws", None), ("c3s", None)])


def test_other_evaluated_networks_small_batch():
    # shapes of the paper's other evaluation networks (Table "Networks description")
    for net in (nets.resnet18(), nets.alexnet(), nets.vgg19(in_hw=64)):
        _net_case(net, 2, [0, 1], False, _plans(net)[:1])


def test_residual_network_with_plain_he_normal_branch_weights():
    """The synthetic residual networks scale the last convolution of every branch by 0.25; here the
    same network with the plain He-normal draw (activations grow with every block, the residual sums
    are large against the branch results), where the kernels' order of operations in the residual
    epilogue -- round the branch result to fp16, add, round -- is furthest from the oracle's single
    fp32 add."""
    from oracle import oracle as o
    net = nets.resnet18()
    x, ws, bs = gen.make_params(net, 2, residual_gain=1.0)
    ref = o.run_net(net, x, ws, bs)
    assert np.abs(ref).max() < 6e4
    s = _session(net, 2, ws, bs)
    try:
        got = s.run_numpy(x)
        compare(got, ref, "resnet18 b2, residual branch gain 1.0")
        _check_groups(s, net, x, ws, bs)
    finally:
        s.close()


def test_run_is_repeatable_and_async_on_a_side_stream():
    from oracle import oracle as o
    net = nets.chain4(32, 28)
    x, ws, bs = gen.make_params(net, 2)
    s = _session(net, 2, ws, bs)
    xt = torch.from_numpy(x).cuda()
    y0 = s.run(xt).clone()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        y1 = s.run(xt)
        y2 = s.run(xt)
    st.synchronize()
    torch.cuda.synchronize()
    assert torch.equal(y0, y1) and torch.equal(y1, y2)
    compare(y0.cpu().numpy(), o.run_net(net, x, ws, bs), "chain4 c32 28x28")
    s.close()


def test_comparison_strategy_plans_compute_the_same_network():
    """Plans of the paper's comparison strategies (no fusion with Eq. 5 budgets, maximal fusion,
    Algorithm 1 with one budget) run through the same kernels and must give the same network."""
    from oracle import oracle as o
    from paper_2011_05630_amd import binding as B
    net = nets.resnet18()
    x, ws, bs = gen.make_params(net, 2)
    ref = o.run_net(net, x, ws, bs)
    for kw in (dict(mode=B.TUNER_LAYERWISE), dict(mode=B.TUNER_LAYERWISE, fixed_budget=32),
               dict(mode=B.TUNER_MAXFUSE), dict(mode=B.TUNER_GREEDY, fixed_budget=64)):
        s = _session(net, 2, ws, bs, **kw)
        try:
            got = s.run_numpy(x)
        finally:
            s.close()
        compare(got, ref, "resnet18 %r" % (kw,))


def test_measured_refinement_keeps_the_results():
    """dlf_plan_refine times alternative tilings of every group and may swap them in: the partition
    stays, and whatever it chose still computes the network."""
    from oracle import oracle as o
    layers = [nets.conv(3, 32, 3, 2, 1, "relu6"), nets.dwconv(32, 3, 1, "relu6"),
              nets.conv(32, 64, 1, 1, 0, "relu6"), nets.dwconv(64, 3, 2, "relu6"),
              nets.conv(64, 128, 1, 1, 0, "relu6"), nets.conv(128, 128, 3, 1, 1, "relu"),
              nets.conv(128, 256, 1, 1, 0, "relu")]
    net = dict(name="refine", layers=layers, in_h=64, in_w=64, in_c=3, input_dist="normal")
    x, ws, bs = gen.make_params(net, 4)
    ref = o.run_net(net, x, ws, bs)
    s = _session(net, 4, ws, bs)
    xt = torch.from_numpy(x).cuda()
    before = [(g["first"], g["last"], g["budget"]) for g in s.groups]
    y0 = s.run(xt).clone()
    torch.cuda.synchronize()
    changed = s.refine(xt, top_k=6, reps=2)
    assert 0 <= changed <= len(before)
    assert [(g["first"], g["last"], g["budget"]) for g in s.groups] == before
    y1 = s.run(xt)
    torch.cuda.synchronize()
    compare(y0.cpu().numpy(), ref, "before refinement")
    compare(y1.cpu().numpy(), ref, "after refinement")
    s.close()


def test_measured_refinement_of_a_bottleneck_block():
    """A whole bottleneck block as one group takes its residual operand from its input; the
    fused-group candidates that dlf_plan_refine times on the same layers take it as a second
    tensor: every candidate must get its own."""
    from oracle import oracle as o
    from paper_2011_05630_amd import binding as B
    layers = [nets.conv(16, 256, 1, 1, 0, "relu"), nets.conv(256, 64, 1, 1, 0, "relu"), nets.conv(64, 64, 3, 1, 1, "relu"),
              nets.conv(64, 256, 1, 1, 0, "relu", residual_from=0), nets.conv(256, 64, 1, 1, 0, "relu")]
    net = dict(name="refine_bneck", layers=layers, in_h=28, in_w=28, in_c=16, input_dist="normal")
    x, ws, bs = gen.make_params(net, 2)
    ref = o.run_net(net, x, ws, bs)
    s = _session(net, 2, ws, bs, mode=B.TUNER_MANUAL, group_last=[0, 3, 4], group_budget=[256] * 3)
    assert B.dlf_plan_group_config(s.plan, 1)["kind"] == 12
    xt = torch.from_numpy(x).cuda()
    changed = s.refine(xt, top_k=4, reps=2)
    assert 0 <= changed <= 3
    y1 = s.run(xt)
    torch.cuda.synchronize()
    compare(y1.cpu().numpy(), ref, "bottleneck block after refinement")
    s.close()


def test_error_paths_return_status_not_crash():
    from paper_2011_05630_amd import binding as B
    net = nets.chain4(256)
    h = B.dlf_net_create(net["layers"], 56, 56, 256)          # shape-only
    with pytest.raises(B.DlfError) as e:
        B.dlf_plan(h, 1, mode=B.TUNER_MANUAL, group_last=[3], group_budget=[64],
                   max_lds_bytes=16 * 1024)
    assert e.value.status == B.DLF_ERR_INFEASIBLE
    p = B.dlf_plan(h, 1)
    x = torch.zeros(1, 56, 56, 256, dtype=torch.float16, device="cuda")
    y = torch.zeros_like(x)
    ws = torch.empty(max(B.dlf_plan_workspace_bytes(p), 256), dtype=torch.uint8, device="cuda")
    B.dlf_plan_bind_workspace(p, ws.data_ptr(), ws.numel())
    with pytest.raises(B.DlfError) as e:
        B.dlf_run(p, x.data_ptr(), y.data_ptr(), None)
    assert e.value.status == 7                                  # no weights
    B.dlf_plan_destroy(p)
    B.dlf_net_destroy(h)


@pytest.mark.gpu
def test_branches_on_a_second_stream_compute_the_same_network():
    """dlf_plan_set_overlap: the projection shortcuts of a residual network on the plan's second
    stream, several runs in a row (each run's buffers are rewritten by the next), against the
    in-order run."""
    import torch
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    net = nets.resnet18()
    batch = 4
    x, ws, bs = gen.make_params(net, batch, 3)
    s = Session(net, batch, ws, bs)
    try:
        n_side = sum(B.dlf_plan_group_stream(s.plan, g) == 1 for g in range(len(s.groups)))
        assert n_side == 0, "in order unless asked for"
        want = s.run_numpy(x)
        B.dlf_plan_set_overlap(s.plan, True)
        n_side = sum(B.dlf_plan_group_stream(s.plan, g) == 1 for g in range(len(s.groups)))
        assert n_side >= 3, "the three projection shortcuts of ResNet-18 do not depend on the layers in front of them"
        xt = torch.from_numpy(x).cuda()
        out = torch.empty(s.out_shape, dtype=torch.float16, device="cuda")
        for _ in range(5):
            s.run(xt, out)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), want)
        B.dlf_plan_set_overlap(s.plan, False)
        assert np.array_equal(s.run_numpy(x), want)
    finally:
        s.close()


@pytest.mark.gpu
def test_a_run_captured_in_a_hip_graph_replays_to_the_eager_result():
    """dlf_run only launches kernels (after its first call on a device), so it can be captured;
    every replay, with eager runs and synchronisations between them, must equal the eager result."""
    from paper_2011_05630_amd.runner import Session
    net = nets.mobilenet_v1()
    batch = 2
    x, ws, bs = gen.make_params(net, batch, 4)
    s = Session(net, batch, ws, bs)
    try:
        xt = torch.from_numpy(x).cuda()
        out = torch.empty(s.out_shape, dtype=torch.float16, device="cuda")
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            s.run(xt, out)                      # first run: one-time kernel set-up, outside the capture
        torch.cuda.synchronize()
        want = out.cpu().numpy().copy()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            s.run(xt, out)
        torch.cuda.synchronize()
        for _ in range(3):
            out.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy(), want)
            s.run(xt, out)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy(), want)
    finally:
        s.close()
