"""Harness of the paper's experiment protocol (Section 6, Appendix "Experimental details"):
host-side constants on the CPU, one run against the oracle on the GPU."""
import math

import numpy as np
import pytest

from oracle import adacgd_oracle as O
from paper_2211_00188_amd import experiments as X
from paper_2211_00188_amd import workloads as W


def test_ef21_constants_closed_forms():
    assert X.ef21_constants(1.0) == (1.0, 0.0)                      # identity compressor: exact
    a, b = X.ef21_constants(0.75)                                   # sqrt(1 - alpha) = 1/2
    assert a == pytest.approx(0.5) and b == pytest.approx(0.5)
    for alpha in (1e-3, 0.04, 0.3):
        a, b = X.ef21_constants(alpha)
        r = math.sqrt(1 - alpha)
        assert a == pytest.approx(1 - r) and b == pytest.approx((1 - alpha) / (1 - r))
        assert b / a == pytest.approx((1 - alpha) / (1 - r) ** 2)
    assert X.three_pc_constants("gd") == (1.0, 0.0)
    assert X.three_pc_constants("lag", zeta=3.0) == (1.0, 3.0)
    assert X.three_pc_constants("clag", [0.75], zeta=3.0) == (pytest.approx(0.5), 3.0)
    a, b = X.three_pc_constants("adacgd", [0.01, 0.75, 0.5], zeta=0.1)
    assert (a, b) == (X.ef21_constants(0.01)[0], X.ef21_constants(0.01)[1])
    assert X.theoretical_stepsize(2.0, 3.0, 1.0, 0.0) == 0.5       # GD: 1 / L


@pytest.mark.parametrize("method", ["lag", "ef21", "clag", "adacgd"])
def test_three_point_inequality_holds_for_the_oracle_compressor(method):
    """||C_{h,y}(x) - x||^2 <= (1 - A) ||h - y||^2 + B ||x - y||^2 (the 3PC property the stepsize
    rule rests on), with the oracle's compressor and points that stress both terms."""
    d = 64
    rng = np.random.default_rng(3)
    levels, zeta = X.method_levels(method, d, adacgd_ratios=(0.05, 0.25, 0.5), zeta=0.7)
    A_, B_ = X.three_pc_constants(method, [k / d for _, k in levels], zeta)
    worst = -np.inf
    for trial in range(400):
        y = rng.standard_normal(d)
        h = y + rng.standard_normal(d) * 10.0 ** rng.uniform(-3, 1)
        x = y + rng.standard_normal(d) * 10.0 ** rng.uniform(-3, 1) * (rng.random(d) < rng.uniform(0.05, 1))
        r = O.adacgd_compress(h.astype(np.float64), y.astype(np.float64), x.astype(np.float64), levels, zeta)
        lhs = float(np.sum((r.h_new - x) ** 2))
        rhs = (1 - A_) * float(np.sum((h - y) ** 2)) + B_ * float(np.sum((x - y) ** 2))
        worst = max(worst, lhs - rhs * (1 + 1e-12))
    assert worst <= 0.0


def test_smoothness_constants_bound_the_gradient_variation():
    wl = W.tiny()
    Lm, Lp = X.smoothness_constants(wl)
    assert 0 < Lm <= Lp * (1 + 1e-12)
    rng = np.random.default_rng(0)
    shards = wl.shards()
    for _ in range(20):
        x, y = rng.standard_normal(wl.d), rng.standard_normal(wl.d)
        gx = np.stack([O.logistic_grad(A, l, x, wl.lam, np.float64) for A, l in shards])
        gy = np.stack([O.logistic_grad(A, l, y, wl.lam, np.float64) for A, l in shards])
        dist2 = float(np.sum((x - y) ** 2))
        assert float(np.sum((gx.mean(0) - gy.mean(0)) ** 2)) <= Lm ** 2 * dist2 * (1 + 1e-9)
        assert float(np.mean(np.sum((gx - gy) ** 2, axis=1))) <= Lp ** 2 * dist2 * (1 + 1e-9)


def test_method_levels_are_the_special_cases():
    d = 300
    assert X.method_levels("gd", d) == ([(W.TOPK, d)], 0.0)
    assert X.method_levels("ef21", d) == ([(W.TOPK, 1)], 0.0)
    assert X.method_levels("clag", d, zeta=2.0) == ([(W.TOPK, 1)], 2.0)
    lv, z = X.method_levels("adacgd", d)
    assert [k for _, k in lv] == [3, 15, 30, 75, 150] and z == 1.0


@pytest.mark.gpu
@pytest.mark.parametrize("method", ["gd", "clag", "adacgd"])
def test_run_matches_oracle_loop(method):
    """The harness's curve (bits per worker, ||grad f||^2) equals the same loop on the oracle."""
    wl = W.tiny()
    levels, zeta = X.method_levels(method, wl.d, zeta=1.0)
    gamma = 0.3
    steps, bits, gn = X.run(wl, method, 1, bit_budget=float("inf"), max_steps=60, chunk=20, base_gamma=gamma)
    orc = O.AdaCGDOracle(n=wl.n, d=wl.d, gamma=gamma, worker_levels=levels, zeta_worker=zeta, master_levels=[],
                         zeta_master=0.0, shards=wl.shards(), lam=wl.lam)
    orc.init(np.zeros(wl.d, dtype=np.float32))
    up = 0
    ref_bits, ref_gn = [0.0], [float(np.sum(orc.y.astype(np.float64).mean(0) ** 2))]
    assert steps.tolist() == [0, 20, 40, 60]
    for t in range(60):
        res, _ = orc.step()
        up += sum(O.AdaCGDOracle.message_bits(r.level, orc.wl, wl.d) for r in res)
        if t + 1 in steps:
            ref_bits.append(up / wl.n)
            ref_gn.append(float(np.sum(orc.y.astype(np.float64).mean(0) ** 2)))
    assert bits.tolist() == ref_bits
    assert np.allclose(gn, ref_gn, rtol=1e-4, atol=0)
    if method == "gd":
        assert bits[-1] == 60 * (1 + wl.d * (32 + 7))      # every coordinate, every step


@pytest.mark.gpu
def test_run_stops_close_to_the_budget():
    wl = W.tiny()
    per_step = 1 + wl.d * (32 + 7)                    # plain gradient descent sends everything
    steps, bits, gn = X.run(wl, "gd", 1, bit_budget=37.5 * per_step, base_gamma=0.3)
    assert steps[-1] == 38 and bits[-1] == 38 * per_step
    assert X.largest_message_bits([(W.TOPK, wl.d)], wl.d) == per_step
