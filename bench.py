#!/usr/bin/env python3
"""Benchmark of the fused-layer CNN executor on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--batch B]
                    [--plan dp|greedy|unfused] [--table] [--no-cpu]

A step is one pass of the whole hot path (every fusion group of the plan) over one batch of
synthetic input that is already resident in HBM.  Prints ONE JSON line: images/s, the roofline
figures of the dominant kernel (measured with HIP events on the launch stream) and the CPU
oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_FP16_PEAK_TFLOPS = 2500.0  # MI355X dense fp16 MFMA
MFMA_INT8_PEAK_TOPS = 5000.0    # MI355X dense int8 MFMA
RIDGE = MFMA_FP16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)   # FLOP per byte

# HBM bytes per launch of a workload's kernels, from two `rocprofv3 --pmc` runs of this file
# (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch; `--calib-copy 3` adds plain 256 MiB device copies
# whose readings give each counter's scale).  `--traffic-from FETCH_DIR WRITE_DIR` turns the two
# counter CSVs into profiles/hbm_traffic.json; the figures are valid only for the kernel sources they
# were taken with (`csrc_sha1`), and `traffic` is reported as null once the sources have changed.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def load_traffic():
    try:
        with open(TRAFFIC_FILE) as f:
            return json.load(f)
    except (OSError, ValueError):
        return {"csrc_sha1": "", "bytes_per_launch": {}}


def kernel_short_name(k):
    k = k.replace("void ", "").split("(")[0].replace(" ", "")
    while k.endswith(",false>"):          # trailing template defaults (second operand pair, quantised form)
        k = k[:-len(",false>")] + ">"
    return k


def traffic_from(fetch_dir, write_dir, workload_key):
    """Reads rocprofv3's counter_collection CSVs of a FETCH_SIZE and a WRITE_SIZE run of
    `bench.py --workload W --calib-copy 3`, scales both counters by what they read for the 256 MiB
    copies, and stores mean HBM bytes per launch of every kernel under `workload_key`.  Prints the
    table that goes into the profile summary."""
    import collections
    import csv
    import glob

    def load(d):
        files = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)
        assert files, "no counter_collection.csv under " + d
        by = collections.defaultdict(list)
        for fn in files:
            for r in csv.DictReader(open(fn)):
                by[r["Kernel_Name"]].append(float(r["Counter_Value"]))
        return by

    F, W = load(fetch_dir), load(write_dir)
    copy = [k for k in F if "copyBuffer" in k or "copy" in k.lower()][0]
    kib = 256 * 1024
    bf, bw = sorted(F[copy])[-3:], sorted(W[copy])[-3:]
    ff, fw = kib / (sum(bf) / len(bf)), kib / (sum(bw) / len(bw))
    rows = []
    for k in F:
        n = kernel_short_name(k)
        if not n.startswith("k_") or k not in W:
            continue
        f, w = sum(F[k]) / len(F[k]), sum(W[k]) / len(W[k])
        rows.append((n, len(F[k]), f, w, int(round((f * ff + w * fw) * 1024))))
    rows.sort(key=lambda r: -r[1] * r[4])
    t = load_traffic()
    if t.get("csrc_sha1") != csrc_sha1():
        t = {"csrc_sha1": csrc_sha1(), "bytes_per_launch": {}}
    t["bytes_per_launch"][workload_key] = {r[0]: r[4] for r in rows}
    t.setdefault("factors", {})[workload_key] = {"FETCH_SIZE": ff, "WRITE_SIZE": fw,
                                                 "copy_readings_KiB": {"FETCH_SIZE": bf, "WRITE_SIZE": bw}}
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(t, f, indent=1, sort_keys=True)
        f.write("\n")
    print("factors: FETCH_SIZE %.4f (%s), WRITE_SIZE %.4f (%s)" % (ff, bf, fw, bw))
    print("| kernel | launches | FETCH_SIZE KiB | WRITE_SIZE KiB | scaled HBM bytes per launch |\n|---|---|---|---|---|")
    for n, cnt, f, w, tot in rows:
        print("| `%s` | %d | %.1f | %.1f | %.1f MB |" % (n, cnt, f, w, tot / 1e6))


def csrc_sha1():
    import hashlib
    h = hashlib.sha1()
    d = os.path.join(ROOT, "paper_2011_05630_amd", "csrc")
    for f in sorted(os.listdir(d)):
        with open(os.path.join(d, f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


VARIANT_NAME = {0: "k_group<2,2,2>", 1: "k_group<1,4,2>", 2: "k_group<1,2,2>", 3: "k_group<1,2,4>"}
# pointwise kernels by item shape
PW_NAME = {0: "k_pw<2,2,6,2>", 1: "k_pw<1,1,8,4>", 2: "k_pw_sk", 3: "k_pwb<2,2>", 4: "k_pwb<1,4>"}
PW2_NAME = {3: "k_pwb<2,2,true>", 4: "k_pwb<1,4,true>"}
DW_NAME = {0: "k_dw<1>", 1: "k_dw<2>"}
C3_NAME = {0: "k_c3b<2,32,2>", 1: "k_c3b<2,64,2>", 2: "k_c3b<1,32,2>", 3: "k_c3b<1,64,2>", 4: "k_c3b<2,32,4>"}


def workloads():
    from synth import nets
    w = {
        "block2": (nets.two_layer_block, 1),
        "vgg16": (nets.vgg16, 16),
        "resnet50": (nets.resnet50, 32),
        "mobilenet_v1": (nets.mobilenet_v1, 64),
        # the other networks of the paper's evaluation (Sec. V, table of networks)
        "vgg19": (nets.vgg19, 16),
        "resnet18": (nets.resnet18, 32),
        "alexnet": (nets.alexnet, 32),
    }
    for c in (16, 32, 64, 128, 256):
        w["chain4_c%d" % c] = ((lambda c=c: nets.chain4(c)), 8)
    return w


def layer_bytes_flops(net, batch):
    """Algorithmic MACs, weight bytes and tensor bytes per layer (Eq. 1/2; fp16 tensors)."""
    from synth import nets
    shapes = nets.infer_shapes(net)
    rows = []
    for L, (hin, hout) in zip(net["layers"], shapes):
        if L["op"] == "conv":
            mac = hout[0] * hout[1] * L["kh"] * L["kw"] * L["cin"] * L["cout"]
            wb = L["cout"] * L["kh"] * L["kw"] * L["cin"] * 2 + 4 * L["cout"]
        elif L["op"] == "dwconv":
            mac = hout[0] * hout[1] * L["kh"] * L["kw"] * L["cout"]
            wb = L["cout"] * L["kh"] * L["kw"] * 2 + 4 * L["cout"]
        elif L["op"] == "fc":
            mac = L["cin"] * L["cout"]
            wb = L["cin"] * L["cout"] * 2 + 4 * L["cout"]
        else:
            mac, wb = 0, 0
        rows.append(dict(mac=mac * batch, wbytes=wb, op=L["op"], k=L["kh"],
                         in_bytes=batch * hin[0] * hin[1] * hin[2] * 2,
                         out_bytes=batch * hout[0] * hout[1] * hout[2] * 2))
    return rows


def group_accounting(net, batch, session):
    """Per fusion group: algorithmic FLOPs and the bytes fusion must move (group input + output +
    weights + residual operand)."""
    from paper_2011_05630_amd import binding as B
    rows = layer_bytes_flops(net, batch)
    out = []
    for g, info in enumerate(session.groups):
        f, l = info["first"], info["last"]
        flops = 2 * sum(rows[i]["mac"] for i in range(f, l + 1))
        flops3x3 = 2 * sum(rows[i]["mac"] for i in range(f, l + 1) if rows[i]["op"] == "conv" and rows[i]["k"] == 3)
        has_dw = any(rows[i]["op"] == "dwconv" for i in range(f, l + 1))
        wbytes = sum(rows[i]["wbytes"] for i in range(f, l + 1))
        in_layer, res_layer = B.dlf_plan_group_io(session.plan, g)
        byts = rows[f]["in_bytes"] + rows[l]["out_bytes"] + wbytes
        cfg = B.dlf_plan_group_config(session.plan, g)
        if cfg["kind"] == 8:
            # projection + last 1x1 layer of a residual block: both inputs (of a strided projection
            # the pixels it uses), one output
            st = net["layers"][f]["stride"]
            byts = rows[f]["in_bytes"] // (st * st) + rows[l]["in_bytes"] + rows[l]["out_bytes"] + wbytes
        elif res_layer >= -1:
            byts += rows[l]["out_bytes"] if res_layer < 0 else rows[res_layer]["out_bytes"]
        if cfg["kind"] == 1:
            kname = "k_fc"
        elif cfg["kind"] == 3:
            kname = PW_NAME[cfg["variant"]]
        elif cfg["kind"] == 2:
            kname = "k_gap"
        elif cfg["kind"] == 4:
            kname = C3_NAME[cfg["variant"]]
        elif cfg["kind"] == 5:
            kname = DW_NAME[cfg["variant"]]
        elif cfg["kind"] == 6:
            kname = "k_dwpw<%d>" % cfg["variant"]
        elif cfg["kind"] == 7:
            kname = "k_dwt<%d>" % (cfg["variant"] + 1)
        elif cfg["kind"] == 10:
            kname = "k_c3s<%d,%d,%d>" % (1 if cfg["variant"] >= 8 else 9, net["layers"][f]["stride"],
                                         2 if info["tile_h"] * info["tile_w"] > 32 else 1)
        elif cfg["kind"] == 12:
            kname = "k_bneck<%d>" % cfg["variant"]
        elif cfg["kind"] == 11:
            kname = "k_c3pw<%d,%d>" % (cfg["variant"], net["layers"][f]["cin"])
        elif cfg["kind"] == 9:
            kname = "k_dws<%d,%d>" % (cfg["variant"] // 2 + 1, cfg["variant"] % 2 + 1)
        elif cfg["kind"] == 8:
            kname = PW2_NAME[cfg["variant"]]         # the same kernel, built for a second operand pair
        else:
            kname = VARIANT_NAME[cfg["variant"]]
        out.append(dict(first=f, last=l, budget=info["budget"], flops=flops, bytes=byts, flops3x3=flops3x3,
                        has_dw=has_dw,
                        kernel=kname, tile=(info["tile_h"], info["tile_w"]), cfg=cfg,
                        model_us=info["model_cost"] / 1e6))
    return out


def time_plan(net, batch, plan, steps, warmup, x=None, ws=None, bs=None, refine=0, calib_copy=0):
    """Builds the session, runs `warmup` untimed and exactly `steps` timed passes of dlf_run between
    two synchronisations, then a profiled pass for per-group durations.  Returns a dict."""
    import torch
    from synth import gen
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    if x is None:
        x, ws, bs = gen.make_params(net, batch)
    s = Session(net, batch, ws, bs, **plan)
    xt = torch.from_numpy(x).cuda()
    out = torch.empty(s.out_shape, dtype=torch.float16, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    if calib_copy > 0:
        src = torch.ones(128 * 1024 * 1024, dtype=torch.float16, device="cuda")     # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(calib_copy):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    refined = s.refine(xt, top_k=refine, reps=5) if refine > 0 else 0
    for _ in range(warmup):
        B.dlf_run(s.plan, xt.data_ptr(), out.data_ptr(), stream)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        B.dlf_run(s.plan, xt.data_ptr(), out.data_ptr(), stream)
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps   # wall clock, sync on both sides
    event_ms_per_step = e0.elapsed_time(e1) / steps
    # per-group durations: a HIP stop event on every group launch, on the launch stream
    reps = max(5, min(50, steps))
    gms = B.dlf_run_profiled(s.plan, xt.data_ptr(), out.data_ptr(), stream, reps)
    # Events stretch the stream: every launch of the profiled pass carries a constant hand-over
    # cost that the timed region (no events) does not have.  It is removed uniformly, so that the
    # group durations add up to the step time measured over the timed region.
    ev_overhead_ms = max(0.0, (sum(gms) - ms_per_step) / len(gms))
    gms = [max(g - ev_overhead_ms, 1e-6) for g in gms]
    acct = group_accounting(net, batch, s)
    for a, ms in zip(acct, gms):
        a["ms"] = ms
    res = dict(ms_per_step=ms_per_step, event_ms_per_step=event_ms_per_step, ev_overhead_ms=ev_overhead_ms,
               acct=acct, groups=len(s.groups), refined=refined, x=x, ws=ws, bs=bs)
    s.close()
    del xt, out
    return res


def class_fractions(net, acct):
    """Roofline fractions of the two classes of groups the targets are stated on.
    mfma: groups whose operations are dominated by 3x3 convolutions and whose intensity lies above
    the ridge -- fraction of the fp16 MFMA peak; depthwise: groups that hold a depthwise layer --
    fraction of the HBM peak on algorithmic bytes.  Each: best group, and all such groups together
    (sum of work / sum of time)."""
    out = {}
    mf = [a for a in acct if a["flops3x3"] * 2 > a["flops"] and a["flops"] / max(a["bytes"], 1) >= RIDGE]
    if mf:
        best = max(mf, key=lambda a: a["flops"] / a["ms"])
        out["mfma_3x3_groups"] = dict(
            groups=len(mf), share_of_step=sum(a["ms"] for a in mf) / sum(a["ms"] for a in acct),
            frac_time_weighted=sum(a["flops"] for a in mf) / (sum(a["ms"] for a in mf) * 1e-3) / 1e12 / MFMA_FP16_PEAK_TFLOPS,
            frac_best=best["flops"] / (best["ms"] * 1e-3) / 1e12 / MFMA_FP16_PEAK_TFLOPS,
            best_group="%d-%d %s" % (best["first"], best["last"], best["kernel"]))
    dw = [a for a in acct if a["has_dw"]]
    if dw:
        best = max(dw, key=lambda a: a["bytes"] / a["ms"])
        out["depthwise_groups"] = dict(
            groups=len(dw), share_of_step=sum(a["ms"] for a in dw) / sum(a["ms"] for a in acct),
            frac_time_weighted=sum(a["bytes"] for a in dw) / (sum(a["ms"] for a in dw) * 1e-3) / 1e9 / HBM_PEAK_GBS,
            frac_best=best["bytes"] / (best["ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
            best_group="%d-%d %s" % (best["first"], best["last"], best["kernel"]))
    return out


def print_table(acct, gms_sum, ms_per_step):
    print("%-10s %-13s %6s %-7s %9s %9s %9s %8s %8s %7s %8s" % (
        "layers", "kernel", "budget", "tile", "us", "model_us", "GFLOP", "MB", "TFLOP/s", "GB/s",
        "roof%"), file=sys.stderr)
    for a in acct:
        t = a["ms"] * 1e-3
        tf = a["flops"] / t / 1e12
        gb = a["bytes"] / t / 1e9
        aig = a["flops"] / max(a["bytes"], 1)
        frac = tf / MFMA_FP16_PEAK_TFLOPS if aig >= RIDGE else gb / HBM_PEAK_GBS
        print("%-10s %-13s %6d %-7s %9.2f %9.2f %9.3f %8.2f %8.1f %7.0f %7.1f%s  s%d x%d lds%dk" % (
            "%d-%d" % (a["first"], a["last"]), a["kernel"], a["budget"],
            "%dx%d" % a["tile"], a["ms"] * 1e3, a["model_us"], a["flops"] / 1e9,
            a["bytes"] / 1e6, tf, gb, 100 * frac, "M" if aig >= RIDGE else "H",
            a["cfg"]["stream0"], a["cfg"]["nslices"], a["cfg"]["lds_bytes"] // 1024),
            file=sys.stderr)
    print("sum of groups %.1f us; step %.1f us" % (gms_sum * 1e3, ms_per_step * 1e3), file=sys.stderr)


def sweep_chain4(steps, warmup):
    """The block-size sweep of Sec. III-B on this chip: chains of four 3x3 convolutions at 56 x 56,
    C -> C for five widths, batch 1 and 8, every fusion depth 1..4 (groups {1,1,1,1}, {2,2}, {3,1},
    {4}) on every CU budget.  One line per point on stdout: feasible?, measured and modelled us,
    fraction of the plan's roofline (sum over groups of max(flops / MFMA peak, bytes / HBM peak))."""
    from synth import nets, gen
    from paper_2011_05630_amd import binding as B
    parts = {1: [0, 1, 2, 3], 2: [1, 3], 3: [2, 3], 4: [3]}
    print("| C | batch | depth | budget | feasible | us | model us | roofline us | fraction |")
    print("|---|---|---|---|---|---|---|---|---|")
    for c in (16, 32, 64, 128, 256):
        net = nets.chain4(c)
        for batch in (1, 8):
            x, ws, bs = gen.make_params(net, batch)
            for depth, lasts in parts.items():
                for budget in (32, 64, 128, 256):
                    plan = dict(mode=B.TUNER_MANUAL, group_last=lasts, group_budget=[budget] * len(lasts))
                    try:
                        r = time_plan(net, batch, plan, steps, warmup, x, ws, bs)
                    except B.DlfError as e:
                        if e.status != B.DLF_ERR_INFEASIBLE:
                            raise
                        print("| %d | %d | %d | %d | no | - | - | - | - |" % (c, batch, depth, budget))
                        continue
                    roof = sum(max(a["flops"] / (MFMA_FP16_PEAK_TFLOPS * 1e12), a["bytes"] / (HBM_PEAK_GBS * 1e9))
                               for a in r["acct"]) * 1e6
                    us = r["ms_per_step"] * 1e3
                    print("| %d | %d | %d | %d | yes | %.1f | %.1f | %.2f | %.3f |" % (
                        c, batch, depth, budget, us, sum(a["model_us"] for a in r["acct"]), roof, roof / us))
                    sys.stdout.flush()


I8_LAYERS = [  # name, batch, h = w, cin, cout, filter: the 3x3 layers of VGG-16 (from 64 channels on) and of the
    # chain of configuration 2, and the 1x1 layers of ResNet-50's bottleneck blocks
    ("vgg_conv1_2", 16, 224, 64, 64, 3), ("vgg_conv2_2", 16, 112, 128, 128, 3), ("vgg_conv3_2", 16, 56, 256, 256, 3),
    ("vgg_conv4_2", 16, 28, 512, 512, 3), ("vgg_conv5_2", 16, 14, 512, 512, 3), ("chain4_c256", 8, 56, 256, 256, 3),
    ("res2_reduce", 32, 56, 256, 64, 1), ("res2_expand", 32, 56, 64, 256, 1), ("res3_reduce", 32, 28, 512, 128, 1),
    ("res3_expand", 32, 28, 128, 512, 1), ("res4_reduce", 32, 14, 1024, 256, 1), ("res4_expand", 32, 14, 256, 1024, 1),
    ("res5_3x3", 32, 7, 512, 512, 3), ("res5_reduce", 32, 7, 2048, 512, 1),
    # a 3x3 layer and the 2x2 max pool behind it as one launch (the last layers of VGG-16's stages 3 and 4)
    ("vgg_conv3_3_pool", 16, 56, 256, 256, 3, True), ("vgg_conv4_3_pool", 16, 28, 512, 512, 3, True),
]


def bench_i8(steps, warmup, cpu=True, layers=None):
    """The quantised (int8) 3x3 layer: us per launch (events on the launch stream around `steps`
    launches back to back), TOP/s by Eq. 1, fraction of the int8 MFMA peak, the same layer in
    fp16 on the block kernel beside it, and the integer oracle on a bounded sample of one layer."""
    import torch
    from synth import gen, nets
    from paper_2011_05630_amd import binding as B
    out = {}
    stream = torch.cuda.current_stream().cuda_stream
    for name, batch, hw, c, co, k, *rest in (layers or I8_LAYERS):
        pool = bool(rest and rest[0])
        ohw = hw // 2 if pool else hw
        x, wt, sc, b = gen.make_i8_layer(batch, hw, hw, c, co, k)
        layer = B.dlf_i8conv_create(batch, hw, hw, c, co, k, True, wt, sc, b, 0, pool)
        info = B.dlf_i8conv_info(layer)
        xt = torch.from_numpy(x).cuda()
        yt = torch.empty((batch, ohw, ohw, co), dtype=torch.int8, device="cuda")
        for _ in range(warmup):
            B.dlf_i8conv_run(layer, xt.data_ptr(), yt.data_ptr(), stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(steps):
            B.dlf_i8conv_run(layer, xt.data_ptr(), yt.data_ptr(), stream)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / steps
        B.dlf_i8conv_destroy(layer)
        tops = info["op_count"] / (us * 1e-6) / 1e12
        nbytes = batch * (hw * hw * c + ohw * ohw * co) + k * k * c * co            # input + output + weights, once each
        rec = dict(batch=batch, hw=hw, cin=c, cout=co, filter=k, pool=pool, us=us, tops=tops,
                   frac_int8_mfma_peak=tops / MFMA_INT8_PEAK_TOPS, gbs=nbytes / (us * 1e-6) / 1e9,
                   frac_hbm_peak=nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                   tile="%dx%d" % (info["th"], info["tw"]), kernel_shape=info["shape"])
        # the same layer in fp16 (one group, the library's own choice of kernel)
        net = dict(name=name, layers=[nets.conv(c, co, k, 1, k // 2, "relu")] + ([nets.maxpool(co, 2, 2, 0)] if pool else []),
                   in_h=hw, in_w=hw, in_c=c, input_dist="normal")
        r = time_plan(net, batch, dict(mode=B.TUNER_DP), steps, warmup)
        assert r["groups"] == 1
        rec["fp16_us"] = r["ms_per_step"] * 1e3
        rec["fp16_kernel"] = r["acct"][0]["kernel"]
        rec["speedup_over_fp16"] = rec["fp16_us"] / us
        out[name] = rec
        del r
    if cpu:
        from oracle import oracle as o
        x, wt, sc, b = gen.make_i8_layer(1, 56, 56, 256, 256, 3)
        t = time.perf_counter()
        o.conv2d_i8(x, wt, sc, b, 1, 1, True)
        dt = time.perf_counter() - t
        out["cpu_baseline"] = dict(value=2 * 56 * 56 * 9 * 256 * 256 / dt / 1e12, unit="TOP/s", cores=o.num_threads(),
                                   kind="oracle", sample="one image of the 56 x 56 x 256 -> 256 layer")
    return out


def bench_i8_vgg_body(steps, warmup, batch=16, hw=224):
    """VGG-16's convolutional body behind its first layer (12 quantised 3x3 layers, the five pools folded
    into the layers in front of them) as a chain of dlf_i8conv_run launches, and the same layers in fp16
    under the DP plan."""
    import torch
    from synth import gen, nets
    from paper_2011_05630_amd import binding as B
    x, params = gen.make_i8_chain(batch, hw)
    stream = torch.cuda.current_stream().cuda_stream
    layers, bufs, ops, h = [], [torch.from_numpy(x).cuda()], 0, hw
    for (wt, sc, b, pool) in params:
        co, ci = wt.shape[0], wt.shape[3]
        layers.append(B.dlf_i8conv_create(batch, h, h, ci, co, 3, True, wt, sc, b, 0, pool))
        ops += B.dlf_i8conv_info(layers[-1])["op_count"]
        h = h // 2 if pool else h
        bufs.append(torch.empty((batch, h, h, co), dtype=torch.int8, device="cuda"))

    def step():
        for l, src, dst in zip(layers, bufs[:-1], bufs[1:]):
            B.dlf_i8conv_run(l, src.data_ptr(), dst.data_ptr(), stream)

    for _ in range(warmup):
        step()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    for l in layers:
        B.dlf_i8conv_destroy(l)
    fl = []
    for (ci, co, pool) in gen.VGG16_BODY:
        fl.append(nets.conv(ci, co, 3, 1, 1, "relu"))
        if pool:
            fl.append(nets.maxpool(co, 2, 2, 0))
    net = dict(name="vgg16_body", layers=fl, in_h=hw, in_w=hw, in_c=64, input_dist="normal")
    r = time_plan(net, batch, dict(mode=B.TUNER_DP), steps, warmup)
    return dict(batch=batch, input="%dx%dx64" % (hw, hw), launches=len(layers), ms_per_step=ms, images_per_s=batch / (ms * 1e-3),
                tops=ops / (ms * 1e-3) / 1e12, frac_int8_mfma_peak=ops / (ms * 1e-3) / 1e12 / MFMA_INT8_PEAK_TOPS,
                fp16_ms_per_step=r["ms_per_step"], fp16_groups=r["groups"], speedup_over_fp16=r["ms_per_step"] / ms)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet50")
    ap.add_argument("--batch", type=int, default=0)
    ap.add_argument("--plan", default="dp", choices=["dp", "greedy", "unfused", "layerwise", "maxfuse"],
                    help="dp: exact minimum of the cost model; greedy: Algorithm 1; unfused: every layer "
                         "alone on --budget CUs; layerwise: every layer alone, budget by Eq. 5; "
                         "maxfuse: longest runnable groups on the largest budget")
    ap.add_argument("--budget", type=int, default=256, help="budget of every group of --plan unfused")
    ap.add_argument("--fixed-budget", type=int, default=0,
                    help="one budget for all groups of --plan greedy / layerwise / maxfuse (0: the tuner's)")
    ap.add_argument("--eq5", default="",
                    help="alpha,beta,scale,offset of Eq. 5 for --plan greedy / layerwise (default: the library's)")
    ap.add_argument("--opcount-critical", type=float, default=0.0,
                    help="Algorithm 1's operation count per CU at which a block is closed (0: the library's)")
    ap.add_argument("--refine", type=int, default=0,
                    help="measured refinement of the plan before timing: candidates per group (0 = off)")
    ap.add_argument("--table", action="store_true", help="per-group table on stderr")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the side measurements (VGG-16 b16, MobileNet-v1 b64, ResNet-50 b1) of the default run")
    ap.add_argument("--sweep", default="", choices=["", "chain4"],
                    help="chain4: the fusion-depth x budget sweep of the 4-layer chains, a table on stdout")
    ap.add_argument("--i8", action="store_true",
                    help="the quantised (int8) 3x3 layer on VGG-16's layer shapes: one JSON line")
    ap.add_argument("--i8-layer", default="", help="with --i8: only this layer (a name of I8_LAYERS)")
    ap.add_argument("--calib-copy", type=int, default=0,
                    help="run this many plain 256 MiB device copies first (reference dispatches of "
                         "known size for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--traffic-from", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"), default=None,
                    help="no GPU: read the counter CSVs of two rocprofv3 --pmc runs of this workload and "
                         "store HBM bytes per launch in profiles/hbm_traffic.json")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU; --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    wl = workloads()
    if args.workload not in wl:
        print("unknown workload %s (have: %s)" % (args.workload, ", ".join(sorted(wl))),
              file=sys.stderr)
        sys.exit(2)
    builder, default_batch = wl[args.workload]
    batch = args.batch or default_batch
    net = builder()
    if args.traffic_from:
        traffic_from(args.traffic_from[0], args.traffic_from[1], "%s_b%d" % (net["name"], batch))
        return
    if args.sweep == "chain4":
        sweep_chain4(min(args.steps, 50), min(args.warmup, 10))
        return
    if args.i8:
        res = {"metric": "int8_conv3x3_tops", "unit": "TOP/s", "dtype": "i8", "data": "synthetic",
               "peak_tops": MFMA_INT8_PEAK_TOPS, "steps": min(args.steps, 100),
               "layers": bench_i8(min(args.steps, 100), min(args.warmup, 10), cpu=not args.no_cpu,
                                  layers=[l for l in I8_LAYERS if l[0] == args.i8_layer] or None)}
        if not args.i8_layer:
            res["vgg16_body_b16"] = bench_i8_vgg_body(min(args.steps, 50), min(args.warmup, 10))
        print(json.dumps(res))
        return

    from paper_2011_05630_amd import binding as B
    n = len(net["layers"])
    if args.plan == "dp":
        plan = dict(mode=B.TUNER_DP)
    elif args.plan == "greedy":
        plan = dict(mode=B.TUNER_GREEDY, fixed_budget=args.fixed_budget)
    elif args.plan == "layerwise":
        plan = dict(mode=B.TUNER_LAYERWISE, fixed_budget=args.fixed_budget)
    elif args.plan == "maxfuse":
        plan = dict(mode=B.TUNER_MAXFUSE, fixed_budget=args.fixed_budget)
    else:
        plan = dict(mode=B.TUNER_MANUAL, group_last=list(range(n)), group_budget=[args.budget] * n)
    if args.plan in ("greedy", "layerwise"):
        if args.eq5:
            al, be, sc, of = (float(v) for v in args.eq5.split(","))
            plan.update(alpha=al, beta=be, mp_scale=sc, mp_offset=of)
        if args.opcount_critical > 0:
            plan.update(opcount_critical=args.opcount_critical)
    r = time_plan(net, batch, plan, args.steps, args.warmup, refine=args.refine, calib_copy=args.calib_copy)
    ms_per_step, acct = r["ms_per_step"], r["acct"]
    x, ws, bs = r["x"], r["ws"], r["bs"]
    gms = [a["ms"] for a in acct]
    images_per_s = batch / (ms_per_step * 1e-3)
    by_kernel = {}
    for a in acct:
        k = by_kernel.setdefault(a["kernel"], dict(ms=0.0, flops=0, bytes=0, launches=0))
        k["ms"] += a["ms"]
        k["flops"] += a["flops"]
        k["bytes"] += a["bytes"]
        k["launches"] += 1
    dom = max(by_kernel, key=lambda k: by_kernel[k]["ms"])
    d = by_kernel[dom]
    ai = d["flops"] / max(d["bytes"], 1)
    avg_ms = d["ms"] / d["launches"]
    if ai >= RIDGE:
        ach = d["flops"] / d["launches"] / (avg_ms * 1e-3) / 1e12
        roof = dict(bound="mfma", achieved=ach, peak=MFMA_FP16_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=ach / MFMA_FP16_PEAK_TFLOPS)
    else:
        ach = d["bytes"] / d["launches"] / (avg_ms * 1e-3) / 1e9
        roof = dict(bound="hbm", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=ach / HBM_PEAK_GBS)
    traffic = None
    tt = load_traffic()
    if tt.get("csrc_sha1") == csrc_sha1():
        traffic = tt["bytes_per_launch"].get("%s_b%d" % (net["name"], batch), {}).get(dom)
    roof.update(traffic=traffic, kernel=dom, launches_per_step=d["launches"],
                avg_launch_us=avg_ms * 1e3, flops_per_launch=d["flops"] / d["launches"],
                bytes_per_launch=d["bytes"] / d["launches"],
                share_of_step=d["ms"] / max(sum(gms), 1e-9))

    if args.table:
        print_table(acct, sum(gms), ms_per_step)

    # Side measurements of the default run: the classes of groups the targets are stated on, in the
    # workloads that have them, and the small batch of the headline network (a few ms each).
    extra = {}
    if not args.no_extra and args.workload == "resnet50" and args.plan == "dp" and not args.batch:
        from synth import nets
        side_steps = max(5, min(args.steps, 50))
        for name, bld, b in (("vgg16_b16", nets.vgg16, 16), ("mobilenet_v1_b64", nets.mobilenet_v1, 64),
                             ("resnet50_b1", nets.resnet50, 1)):
            sn = bld()
            sr = time_plan(sn, b, dict(mode=B.TUNER_DP), side_steps, min(args.warmup, 10))
            e = dict(images_per_s=b / (sr["ms_per_step"] * 1e-3), ms_per_step=sr["ms_per_step"], groups=sr["groups"],
                     steps=side_steps)
            tot = sum(max(a["flops"] / (MFMA_FP16_PEAK_TFLOPS * 1e12), a["bytes"] / (HBM_PEAK_GBS * 1e9)) for a in sr["acct"])
            e["whole_step_roofline_frac"] = tot / (sr["ms_per_step"] * 1e-3)
            e.update(class_fractions(sn, sr["acct"]))
            extra[name] = e
            if args.table:
                print("--- %s" % name, file=sys.stderr)
                print_table(sr["acct"], sum(a["ms"] for a in sr["acct"]), sr["ms_per_step"])
            del sr
        i8 = bench_i8(side_steps, min(args.warmup, 10), cpu=False, layers=[I8_LAYERS[2]])
        extra["i8_conv3x3_256_56x56_b16"] = i8[I8_LAYERS[2][0]]
        extra["i8_vgg16_body_b16"] = bench_i8_vgg_body(side_steps, min(args.warmup, 10))

    cpu = None
    if not args.no_cpu:
        from oracle import oracle as o
        nsample = 1
        t = time.perf_counter()
        o.run_net(net, x[:1], ws, bs)
        dt1 = time.perf_counter() - t
        if dt1 < 5.0:
            nsample = int(max(1, min(batch, 15.0 // max(dt1, 1e-3))))
            t = time.perf_counter()
            o.run_net(net, x[:nsample], ws, bs)
            dt = time.perf_counter() - t
        else:
            dt = dt1
        cpu = dict(value=nsample / dt, unit="images/s", cores=o.num_threads(), kind="oracle",
                   sample="%d image(s) of the same seeded batch, whole network, fp32 nested loops"
                          % nsample)

    total_flops = sum(a["flops"] for a in acct)
    whole = sum(max(a["flops"] / (MFMA_FP16_PEAK_TFLOPS * 1e12), a["bytes"] / (HBM_PEAK_GBS * 1e9)) for a in acct)
    res = {
        "metric": "images_per_sec", "value": images_per_s, "unit": "images/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "%s_b%d" % (net["name"], batch), "batch": batch,
                   "plan": args.plan + ("@%d" % args.fixed_budget if args.fixed_budget > 0 else "")
                   + ("[eq5 %s]" % args.eq5 if args.eq5 and args.plan in ("greedy", "layerwise") else "")
                   + ("[crit %g]" % args.opcount_critical if args.opcount_critical > 0 and args.plan == "greedy" else "")
                   + ("@%d" % args.budget if args.plan == "unfused" else "")
                   + ("+refine%d" % args.refine if args.refine > 0 else ""),
                   "groups_refined": r["refined"], "groups": r["groups"], "layers": n,
                   "input": "%dx%dx%d" % (net["in_h"], net["in_w"], net["in_c"])},
        "event_ms_per_step": r["event_ms_per_step"],
        "event_overhead_us_per_launch": r["ev_overhead_ms"] * 1e3,
        "algorithmic_tflops": total_flops / (ms_per_step * 1e-3) / 1e12,
        "whole_step_roofline_frac": whole / (ms_per_step * 1e-3),
        "roofline": roof, "cpu_baseline": cpu,
    }
    res.update(class_fractions(net, acct))
    if extra:
        res["other_workloads"] = extra
    print(json.dumps(res))


if __name__ == "__main__":
    main()
