"""Characterisation of single convolution layers on the GPU, after the paper's Sec. III-A / III-B
and Sec. IV-A: how achieved GFLOP/s depends on a layer's operation count and channel count with
few and with many compute units, the operation count at which it saturates (OpCount_critical), the
smallest CU budget that reaches a layer's best time, and a least-squares fit of Eq. 5's constants
to those budgets.

Every measurement runs the layer through libdlf (one group, the given budget); this module only
builds layer lists, calls the library and does the regression.

    python -m paper_2011_05630_amd.characterize [--out FILE.json] [--quick]
"""
import argparse
import json
import math
import sys

import numpy as np

BUDGETS = (8, 16, 32, 64, 128, 256)
SMALL_BUDGET = 8          # 1/32 of the chip: the analogue of one of the paper's 32 cores


def conv_ops(cin, cout, hw, k, batch=1):
    """Operation count of the layer {cin, cout, hw x hw, k x k} (stride 1, 'same' padding) as the
    library reports it for a shape-only network (dlf_net_layer_info: Eq. 1), times the batch."""
    from . import binding as B
    layer = dict(op="conv", cin=cin, cout=cout, kh=k, kw=k, stride=1, pad=k // 2, has_bias=1,
                 act="relu", input_from=-1, residual_from=-1)
    h = B.dlf_net_create([layer], hw, hw, cin)
    try:
        return batch * B.dlf_net_layer_info(h, 0)[3]
    finally:
        B.dlf_net_destroy(h)


# ----------------------------------------------------------------------------------------------
# Pure arithmetic (no GPU): saturation point, smallest sufficient budget, Eq. 5 fit
# ----------------------------------------------------------------------------------------------

def opcount_critical(ops, gflops, frac=0.9):
    """Smallest operation count whose layers reach `frac` of the best rate seen at any larger or
    equal count (Sec. III-A: beyond it the rate no longer rises).  ops, gflops: sequences."""
    order = np.argsort(ops)
    o = np.asarray(ops, dtype=np.float64)[order]
    g = np.asarray(gflops, dtype=np.float64)[order]
    top = g.max()
    for i in range(len(o)):
        if g[i] >= frac * top:
            return float(o[i])
    return float(o[-1])


def sufficient_budget(times_by_budget, tol=0.05):
    """Smallest budget whose time is within `tol` of the layer's best time (dict budget -> time)."""
    best = min(times_by_budget.values())
    for b in sorted(times_by_budget):
        if times_by_budget[b] <= (1.0 + tol) * best:
            return b
    return max(times_by_budget)


def fit_eq5(channels, ops, mps):
    """Least squares for MP = a_c * log2(C) + a_o * log2(OpCount) + b  (Eq. 5 read as MP = k *
    (alpha log2 C + beta log2 OpCount) + b).  Returns alpha, beta (normalised to alpha + beta = 1),
    k = a_c + a_o, b and the coefficient of determination."""
    x = np.stack([np.log2(np.asarray(channels, dtype=np.float64)),
                  np.log2(np.asarray(ops, dtype=np.float64)),
                  np.ones(len(mps))], axis=1)
    y = np.asarray(mps, dtype=np.float64)
    coef, _, _, _ = np.linalg.lstsq(x, y, rcond=None)
    a_c, a_o, b = coef
    pred = x @ coef
    ss_res = float(((y - pred) ** 2).sum())
    ss_tot = float(((y - y.mean()) ** 2).sum())
    k = a_c + a_o
    return dict(a_c=float(a_c), a_o=float(a_o),
                alpha=float(a_c / k) if k != 0 else float("nan"),
                beta=float(a_o / k) if k != 0 else float("nan"),
                k=float(k), b=float(b), r2=1.0 - ss_res / ss_tot if ss_tot > 0 else 1.0)


def fit_scale(channels, ops, mps, alpha=0.316, beta=0.659):
    """Least squares for the proportionality constants of Eq. 5 with its weights as printed:
    MP = k * (alpha log2 C + beta log2 OpCount) + b.  Returns k, b and R^2."""
    score = alpha * np.log2(np.asarray(channels, dtype=np.float64)) + beta * np.log2(np.asarray(ops, dtype=np.float64))
    x = np.stack([score, np.ones(len(mps))], axis=1)
    y = np.asarray(mps, dtype=np.float64)
    coef, _, _, _ = np.linalg.lstsq(x, y, rcond=None)
    pred = x @ coef
    ss_res = float(((y - pred) ** 2).sum())
    ss_tot = float(((y - y.mean()) ** 2).sum())
    return dict(k=float(coef[0]), b=float(coef[1]), r2=1.0 - ss_res / ss_tot if ss_tot > 0 else 1.0)


def influence(rows, keys=("log2_ops", "log2_c", "k", "log2_hw")):
    """|Pearson correlation| of log2(GFLOP/s) with each layer parameter over a sweep: the ranking the
    paper takes from its PCA (operation count first, channel second on its chip)."""
    y = np.log2(np.asarray([r["gflops"] for r in rows], dtype=np.float64))
    out = {}
    for key in keys:
        x = np.asarray([r[key] for r in rows], dtype=np.float64)
        if x.std() == 0 or y.std() == 0:
            out[key] = 0.0
        else:
            out[key] = float(abs(np.corrcoef(x, y)[0, 1]))
    return out


# ----------------------------------------------------------------------------------------------
# Measurement (needs the GPU and the built library)
# ----------------------------------------------------------------------------------------------

def _layer(cin, cout, k):
    from synth import nets
    return nets.conv(cin, cout, k, 1, k // 2, "relu")


def time_layer(cin, cout, hw, k, budget, batch=1, reps=5, seed=1):
    """Mean time in seconds of one launch of the layer as its own group on `budget` CUs."""
    import torch
    from synth import gen
    from . import binding as B
    from .runner import Session
    net = dict(name="layer", layers=[_layer(cin, cout, k)], in_h=hw, in_w=hw, in_c=cin,
               input_dist="normal")
    x, ws, bs = gen.make_params(net, batch, seed)
    s = Session(net, batch, ws, bs, mode=B.TUNER_MANUAL, group_last=[0], group_budget=[budget])
    try:
        xt = torch.from_numpy(x).cuda()
        out = torch.empty(s.out_shape, dtype=torch.float16, device="cuda")
        stream = torch.cuda.current_stream().cuda_stream
        B.dlf_run_profiled(s.plan, xt.data_ptr(), out.data_ptr(), stream, 2)     # warm-up
        ms = B.dlf_run_profiled(s.plan, xt.data_ptr(), out.data_ptr(), stream, reps)[0]
    finally:
        s.close()
    return ms * 1e-3


def _row(cin, cout, hw, k, budget, t):
    ops = conv_ops(cin, cout, hw, k)
    return dict(cin=cin, cout=cout, hw=hw, k=k, budget=budget, seconds=t, ops=ops,
                gflops=ops / t / 1e9, log2_ops=math.log2(ops), log2_c=math.log2(min(cin, cout)),
                log2_hw=math.log2(hw))


def run(quick=False, log=sys.stderr):
    """All sweeps; returns a dict of rows and derived figures."""
    max_small_ops = 4e9 if quick else 2e10       # keeps a launch on 8 CUs below about a second
    res = {}

    # (a) few CUs: rate against operation count (channels x feature sizes, 3x3 and 1x1)
    rows = []
    chans = (16, 64, 256) if quick else (16, 32, 64, 128, 256, 512)
    sizes = (14, 56) if quick else (14, 28, 56, 112, 224)
    for k in (3, 1):
        for c in chans:
            for hw in sizes:
                if conv_ops(c, c, hw, k) > max_small_ops:
                    continue
                rows.append(_row(c, c, hw, k, SMALL_BUDGET, time_layer(c, c, hw, k, SMALL_BUDGET)))
                print("few-CU", rows[-1]["cin"], hw, k, "%.1f GFLOP/s" % rows[-1]["gflops"], file=log, flush=True)
    res["few_cu"] = rows
    res["opcount_critical_few_cu"] = opcount_critical([r["ops"] for r in rows], [r["gflops"] for r in rows])
    res["opcount_critical_per_cu"] = res["opcount_critical_few_cu"] / SMALL_BUDGET
    res["influence_few_cu"] = influence(rows)

    # (b) one parameter at a time around {64, 64, 56x56, 3x3}
    rows = []
    for c in ((16, 64, 256) if quick else (16, 32, 64, 128, 256, 512)):
        rows.append(dict(vary="channel", **_row(c, c, 56, 3, SMALL_BUDGET, time_layer(c, c, 56, 3, SMALL_BUDGET))))
    for k in ((1, 3) if quick else (1, 3, 5, 7)):
        rows.append(dict(vary="kernel", **_row(64, 64, 56, k, SMALL_BUDGET, time_layer(64, 64, 56, k, SMALL_BUDGET))))
    for hw in ((14, 56) if quick else (14, 28, 56, 112, 224)):
        rows.append(dict(vary="feature", **_row(64, 64, hw, 3, SMALL_BUDGET, time_layer(64, 64, hw, 3, SMALL_BUDGET))))
    res["one_parameter"] = rows

    # (c) many CUs: {64 f, 64 f, 224 x 224, 3 x 3} over the budgets; (d) three layers of equal count
    layers = [(16, 224), (32, 224), (64, 224), (128, 224)] if not quick else [(16, 224), (64, 224)]
    layers += [(32, 224), (64, 112), (128, 56)]
    if not quick:
        layers += [(64, 56), (64, 14), (256, 14), (256, 28), (512, 7), (512, 14), (16, 56), (128, 28), (32, 28)]
    seen, rows = set(), []
    for c, hw in layers:
        if (c, hw) in seen:
            continue
        seen.add((c, hw))
        times = {}
        for b in BUDGETS:
            times[b] = time_layer(c, c, hw, 3, b)
            rows.append(_row(c, c, hw, 3, b, times[b]))
        print("budgets", c, hw, " ".join("%d:%.1fus" % (b, times[b] * 1e6) for b in BUDGETS), file=log, flush=True)
    res["budget_sweep"] = rows
    per_layer = {}
    for r in rows:
        per_layer.setdefault((r["cin"], r["hw"]), {})[r["budget"]] = r["seconds"]
    fit_rows = []
    for (c, hw), times in sorted(per_layer.items()):
        fit_rows.append(dict(c=c, hw=hw, ops=conv_ops(c, c, hw, 3), sufficient_budget=sufficient_budget(times),
                             best_budget=min(times, key=times.get)))
    res["sufficient_budget"] = fit_rows
    res["eq5_fit"] = fit_eq5([r["c"] for r in fit_rows], [r["ops"] for r in fit_rows],
                             [r["sufficient_budget"] for r in fit_rows])
    res["eq5_scale_fit"] = fit_scale([r["c"] for r in fit_rows], [r["ops"] for r in fit_rows],
                                     [r["sufficient_budget"] for r in fit_rows])
    return res


def summary(res):
    lines = []
    lines.append("few-CU sweep (%d CUs): %d layers, OpCount_critical %.3g operations (%.3g per CU)" % (
        SMALL_BUDGET, len(res["few_cu"]), res["opcount_critical_few_cu"], res["opcount_critical_per_cu"]))
    lines.append("influence on log2(GFLOP/s), |r|: " + ", ".join(
        "%s %.2f" % kv for kv in sorted(res["influence_few_cu"].items(), key=lambda kv: -kv[1])))
    for vary in ("channel", "kernel", "feature"):
        rs = [r for r in res["one_parameter"] if r["vary"] == vary]
        key = dict(channel="cin", kernel="k", feature="hw")[vary]
        lines.append("vary %s: " % vary + ", ".join("%d: %.0f" % (r[key], r["gflops"]) for r in rs) + " GFLOP/s")
    for r in res["sufficient_budget"]:
        lines.append("{%d, %d, %dx%d, 3x3}: %.3g operations, sufficient budget %d, fastest at %d" % (
            r["c"], r["c"], r["hw"], r["hw"], r["ops"], r["sufficient_budget"], r["best_budget"]))
    f = res["eq5_fit"]
    lines.append("free fit: MP = %.1f log2(C) + %.1f log2(OpCount) + %.1f (R^2 %.2f)" % (f["a_c"], f["a_o"], f["b"], f["r2"]))
    g = res["eq5_scale_fit"]
    lines.append("Eq. 5 with alpha 0.316, beta 0.659: MP = %.1f * score + %.1f (R^2 %.2f)" % (g["k"], g["b"], g["r2"]))
    return "\n".join(lines)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default="")
    ap.add_argument("--quick", action="store_true", help="a few layers only")
    a = ap.parse_args()
    res = run(quick=a.quick)
    print(summary(res))
    if a.out:
        with open(a.out, "w") as fh:
            json.dump(res, fh, indent=1)


if __name__ == "__main__":
    main()
