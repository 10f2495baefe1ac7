"""The characterisation tool (Sec. III-A / IV-A sweeps): its arithmetic on the CPU, one small
measurement on the GPU."""
import math

import numpy as np
import pytest

from paper_2011_05630_amd import characterize as ch


def test_operation_count_is_eq1_times_two():
    # {64, 64, 224 x 224, 3 x 3}: 224^2 * 9 * 64 * 64 multiply-adds
    assert ch.conv_ops(64, 64, 224, 3) == 2 * 224 * 224 * 9 * 64 * 64
    # the three layers of Sec. IV-A have the same count
    a, b, c = ch.conv_ops(32, 32, 224, 3), ch.conv_ops(64, 64, 112, 3), ch.conv_ops(128, 128, 56, 3)
    assert a == b == c


def test_eq5_fit_recovers_known_constants():
    rng = np.random.default_rng(0)
    chans = 2 ** rng.integers(4, 10, size=40)
    ops = 2.0 ** rng.uniform(20, 36, size=40)
    alpha, beta, k, b = 0.316, 0.659, 64.0, -1056.0
    # Eq. 5 with alpha + beta = 0.975 as printed: the fit normalises the pair to sum 1
    mp = k * (alpha * np.log2(chans) + beta * np.log2(ops)) + b
    f = ch.fit_eq5(chans, ops, mp)
    assert abs(f["alpha"] - alpha / (alpha + beta)) < 1e-9
    assert abs(f["beta"] - beta / (alpha + beta)) < 1e-9
    assert abs(f["k"] - k * (alpha + beta)) < 1e-6
    assert abs(f["b"] - b) < 1e-6
    assert f["r2"] > 1 - 1e-12
    g = ch.fit_scale(chans, ops, mp)
    assert abs(g["k"] - k) < 1e-6 and abs(g["b"] - b) < 1e-5 and g["r2"] > 1 - 1e-12


def test_saturation_point_and_sufficient_budget():
    ops = [1e6, 1e7, 1e8, 1e9, 1e10]
    gf = [10.0, 100.0, 800.0, 950.0, 1000.0]
    assert ch.opcount_critical(ops, gf, frac=0.9) == 1e9
    assert ch.opcount_critical(ops[::-1], gf[::-1], frac=0.75) == 1e8      # order of the rows is free
    times = {8: 10.0, 16: 5.2, 32: 5.0, 64: 4.9, 128: 4.9, 256: 5.1}
    assert ch.sufficient_budget(times, tol=0.05) == 32
    assert ch.sufficient_budget(times, tol=0.10) == 16
    assert ch.sufficient_budget({8: 1.0, 256: 1.0}) == 8


def test_influence_ranks_the_driving_parameter_first():
    rows = []
    for c in (16, 64, 256):
        for hw in (14, 56):
            ops = ch.conv_ops(c, c, hw, 3)
            rows.append(dict(gflops=ops ** 0.5, log2_ops=math.log2(ops), log2_c=math.log2(c), k=3,
                             log2_hw=math.log2(hw)))
    inf = ch.influence(rows)
    assert inf["log2_ops"] > 0.999 and inf["k"] == 0.0
    assert inf["log2_ops"] >= inf["log2_c"] and inf["log2_ops"] >= inf["log2_hw"]


@pytest.mark.gpu
def test_one_layer_is_timed_on_two_budgets():
    t8 = ch.time_layer(32, 32, 28, 3, 8, reps=3)
    t256 = ch.time_layer(32, 32, 28, 3, 256, reps=3)
    assert 0 < t256 <= t8 * 1.5 and t8 < 1e-2
