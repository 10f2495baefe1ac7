"""The host side of the library (shape checking, cost model, tuners, plan queries, argument
checking) under AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU.

tests/host_sanitize_driver.cpp is compiled together with csrc/dlf_host.cpp, host code instrumented,
the kernel launchers replaced by stand-ins that abort if reached; it replays a script of C-ABI calls
on shape-only networks.  A sanitizer report ends the driver with a non-zero status.  The plans it
prints are compared with those of the ordinary build, so the instrumented run is known to have
walked the same code."""
import os
import random
import re
import subprocess

import pytest

from synth import nets
from paper_2011_05630_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BUDGETS = (32, 64, 128, 256)


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    d = tmp_path_factory.mktemp("san")
    exe = str(d / "host_sanitize_driver")
    host = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
            "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    cmd = (["hipcc", "-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "-x", "hip"] + host +
           ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
            "-o", exe, os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"),
            os.path.join(ROOT, "paper_2011_05630_amd", "csrc", "dlf_host.cpp")])
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout
    return exe


def _net_lines(net):
    out = ["net %d %d %d %d" % (net["in_h"], net["in_w"], net["in_c"], len(net["layers"]))]
    for L in net["layers"]:
        out.append(" ".join(str(v) for v in (
            B.OP[L["op"]], L["cin"], L["cout"], L["kh"], L["kw"], L["stride"], L["pad"], L["has_bias"],
            B.ACT[L["act"]], L["input_from"], L["residual_from"])))
    return out


def _run(exe, lines):
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([exe], input="\n".join(lines) + "\n", stdout=subprocess.PIPE, stderr=subprocess.PIPE,
                       text=True, env=env, timeout=600)
    assert r.returncode == 0, "status %d\n%s\n%s" % (r.returncode, r.stdout[-2000:], r.stderr[-6000:])
    assert "runtime error" not in r.stderr and "Sanitizer" not in r.stderr, r.stderr[-6000:]
    return r.stdout.splitlines()


def _groups_of(line):
    return [(int(a), int(b), int(c)) for a, b, c in re.findall(r"\[(\d+),(\d+)\]@(\d+)", line)]


def _library_groups(net, batch, mode):
    h = B.dlf_net_create(net["layers"], net["in_h"], net["in_w"], net["in_c"])
    p = B.dlf_plan(h, batch, mode=mode, budgets=list(BUDGETS))
    gs = [(g["first"], g["last"], g["budget"]) for g in B.dlf_plan_groups(p)]
    B.dlf_plan_destroy(p)
    B.dlf_net_destroy(h)
    return gs


WORKLOADS = [
    (nets.vgg16(), 16), (nets.resnet50(), 32), (nets.mobilenet_v1(), 64), (nets.resnet18(), 32),
    (nets.alexnet(), 8), (nets.vgg19(in_hw=64), 2), (nets.identical_chain(64, 56, 8), 4),
    (nets.identical_chain(512, 14, 4), 1), (nets.chain4(32), 1), (nets.two_layer_block(), 1),
    (nets.mobilenet_v1(in_hw=64, nblocks=5), 3),
]


def test_planner_under_sanitizers(driver):
    modes = (B.TUNER_DP, B.TUNER_GREEDY, B.TUNER_LAYERWISE, B.TUNER_MAXFUSE)
    lines, expect = [], []
    for net, batch in WORKLOADS:
        lines += _net_lines(net)
        for m in modes:
            lines.append("plan %d %d 0 0" % (batch, m))
            expect.append((net, batch, m))
        lines.append("plan %d %d 64 0" % (batch, B.TUNER_GREEDY))          # fixed budget
        lines.append("plan %d %d 0 %d" % (batch, B.TUNER_DP, 64 * 1024))   # a smaller on-chip memory
        lines.append("manual %d 1 %d 64" % (batch, len(net["layers"]) - 1))  # whole net as one group
        lines.append("manual %d 2 3 64 1 64" % batch)                       # group ends out of order
        lines.append("costs %d" % batch)
        lines.append("badargs")
    out = _run(driver, lines)
    plans = [l for l in out if l.startswith("plan ") and "groups:" in l]
    # the default-option plans come first for each net, in the order of `modes`
    per_net = len(modes) + 2
    assert len(plans) == per_net * len(WORKLOADS), "\n".join(out[-40:])
    for i, (net, batch, m) in enumerate(expect):
        line = plans[(i // len(modes)) * per_net + i % len(modes)]
        assert _groups_of(line) == _library_groups(net, batch, m), (net["name"], batch, m, line)
    assert sum(l.startswith("costs ") for l in out) == len(WORKLOADS)
    assert sum(l == "badargs rejected" for l in out) == len(WORKLOADS)


def test_random_and_malformed_nets_under_sanitizers(driver):
    rng = random.Random(20251)
    lines = []
    n_bad = 0
    for t in range(60):
        c = rng.choice([3, 8, 16, 24, 32, 64, 96])
        hw = rng.choice([7, 14, 20, 28, 33])
        layers = []
        cin = c
        for i in range(rng.randint(1, 9)):
            kind = rng.choice(["c3", "c1", "dw", "pool", "c3s2", "c5", "fc", "gap"])
            if kind == "c3":
                cout = rng.choice([16, 32, 48, 64])
                layers.append(nets.conv(cin, cout, 3, 1, 1, "relu"))
            elif kind == "c5":
                cout = rng.choice([16, 32])
                layers.append(nets.conv(cin, cout, 5, 1, 2, "relu"))
            elif kind == "c3s2":
                cout = rng.choice([32, 64])
                layers.append(nets.conv(cin, cout, 3, 2, 1, "relu"))
            elif kind == "c1":
                cout = rng.choice([16, 32, 64, 128])
                layers.append(nets.conv(cin, cout, 1, 1, 0, rng.choice(["relu", "none", "relu6"])))
            elif kind == "dw":
                cout = cin
                layers.append(nets.dwconv(cin, 3, rng.choice([1, 2])))
            elif kind == "pool":
                cout = cin
                layers.append(nets.maxpool(cin, rng.choice([2, 3]), 2, rng.choice([0, 1])))
            elif kind == "gap":
                cout = cin
                layers.append(nets.gavgpool(cin))
            else:
                cout = rng.choice([10, 100])
                layers.append(nets.fc(cin, cout))      # cin is wrong unless the map is 1x1: rejected by shape check
            cin = cout
        if rng.random() < 0.3 and len(layers) >= 3:      # a residual edge, legal or not
            layers[-1]["residual_from"] = rng.randrange(-1, len(layers))
        if rng.random() < 0.1:                           # a field out of range
            L = rng.choice(layers)
            L[rng.choice(["cin", "cout", "kh", "stride", "pad"])] = rng.choice([-1, 0, 1 << 30])
            n_bad += 1
        net = dict(name="r%d" % t, layers=layers, in_h=hw, in_w=hw, in_c=c, input_dist="uniform")
        lines += _net_lines(net)
        # every command after a rejected net would stop the driver: plan only if the ordinary build accepts it
        try:
            h = B.dlf_net_create(layers, hw, hw, c)
        except B.DlfError:
            continue
        B.dlf_net_destroy(h)
        for m in (B.TUNER_DP, B.TUNER_GREEDY, B.TUNER_LAYERWISE, B.TUNER_MAXFUSE):
            lines.append("plan %d %d 0 0" % (rng.choice([1, 2, 5, 32]), m))
        lines.append("costs %d" % rng.choice([1, 3]))
    out = _run(driver, lines)
    assert sum(l.startswith("net ") for l in out) == 60
    assert any(l.startswith("net ") and not l.endswith(": ok") for l in out)
    assert sum(l.startswith("plan ") for l in out) >= 40
