"""Pins for the oracle's AdaCGD compressor (Section 4.3), the special cases the
paper names (EF21, CLAG, LAG, plain gradient descent), the objective of
Section 6 and the per-step invariants of Algorithms 1 and 2.  CPU only."""
import math

import numpy as np
import pytest

from oracle import adacgd_oracle as O
from paper_2211_00188_amd import workloads as W

T = O.TOPK


# ------------------------------------------------------------ cascade
def _case(tau_target):
    """v = (4,3,2,1): S = 30, Top-1/2/3 errors 14, 5, 1.  D = tau_target with zeta = 1."""
    h = np.array([1, -1, 2, 0.5], dtype=np.float64)
    v = np.array([4, -3, 2, -1], dtype=np.float64)
    x = h + v
    w = np.zeros(4)
    w[0] = math.sqrt(tau_target)
    y = x - w
    return h, y, x


@pytest.mark.parametrize("tau,expect", [
    (36.0, 0), (30.25, 0),           # ||x-h||^2 <= tau  -> keep h (skip)
    (25.0, 1), (16.0, 1),            # first level whose realised error fits
    (12.25, 2), (6.25, 2),
    (4.0, 3), (0.25, 3), (0.0, 3),   # nothing fits -> last level, even though its error is 1 > tau
])
def test_cascade_decision_table(tau, expect):
    h, y, x = _case(tau)
    r = O.adacgd_compress(h, y, x, [(T, 1), (T, 2), (T, 3)], 1.0)
    assert (r.S, r.err) == (30.0, [14.0, 5.0, 1.0])
    assert r.D == tau
    assert r.level == expect
    if expect == 0:
        assert np.array_equal(r.h_new, h) and r.msg_idx.size == 0
    else:
        assert r.msg_idx.tolist() == list(range(expect))
        assert np.array_equal(r.h_new[:expect], x[:expect]) and np.array_equal(r.h_new[expect:], h[expect:])


def test_cascade_boundary_equalities_accept():
    # Eq. (10) and the first branch use "<=": exact equality accepts.
    for D, expect in [(30.0, 0), (14.0, 1), (5.0, 2)]:
        h = np.zeros(4)
        x = np.array([4.0, -3, 2, -1])
        y = x.copy()
        y[1] -= 0  # D is passed directly below
        r = O.adacgd_compress(h, None, None, [(T, 1), (T, 2), (T, 3)], 1.0, D_given=D, v_given=x)
        assert r.level == expect
    # zeta scales the right side
    r = O.adacgd_compress(np.zeros(4), None, None, [(T, 1), (T, 2), (T, 3)], 0.5, D_given=28.0,
                          v_given=np.array([4.0, -3, 2, -1]))
    assert r.level == 1


def test_realised_error_bound_of_adaptive_compressor():
    # Lemma 2 / the definition: the branch taken has error <= max(zeta D, (1 - alpha_m) ||v||^2).
    rng = np.random.default_rng(21)
    d = 200
    levels = [(T, 1), (T, 5), (T, 20), (T, 100)]
    for trial in range(60):
        h = rng.standard_normal(d).astype(np.float32)
        x = (h + rng.standard_normal(d) * 10.0 ** rng.uniform(-2, 1)).astype(np.float32)
        y = (x + rng.standard_normal(d) * 10.0 ** rng.uniform(-2, 1)).astype(np.float32)
        zeta = float(10.0 ** rng.uniform(-2, 1))
        r = O.adacgd_compress(h, y, x, levels, zeta)
        realised = O.sum_sq_diff(x, r.h_new)
        bound = max(np.float64(np.float32(zeta)) * r.D, (1 - 100 / d) * r.S)
        assert realised <= bound * (1 + 1e-6)
        if 0 < r.level < len(levels):
            assert r.err[r.level - 1] <= np.float64(np.float32(zeta)) * r.D
            assert all(e > np.float64(np.float32(zeta)) * r.D for e in r.err[:r.level - 1])
            assert r.S > np.float64(np.float32(zeta)) * r.D


# ------------------------------------------------------------ objective
def test_gradient_closed_form_at_zero_and_finite_differences():
    rng = np.random.default_rng(31)
    N, d, lam = 40, 13, 0.1
    A = rng.standard_normal((N, d)).astype(np.float32)
    yl = np.where(rng.random(N) < 0.5, 1.0, -1.0).astype(np.float32)
    g0 = O.logistic_grad(A, yl, np.zeros(d), lam, np.float64)
    ref0 = -(yl.astype(np.float64)[:, None] * A.astype(np.float64)).sum(0) / (2 * N)
    assert np.allclose(g0, ref0, rtol=1e-13, atol=1e-15)
    x = rng.standard_normal(d)
    g = O.logistic_grad(A, yl, x, lam, np.float64)
    eps = 1e-6
    for j in range(d):
        e = np.zeros(d)
        e[j] = eps
        fd = (O.logistic_loss(A, yl, x + e, lam) - O.logistic_loss(A, yl, x - e, lam)) / (2 * eps)
        assert abs(fd - g[j]) < 1e-8
    # regulariser alone: no data term when labels cancel
    A2 = np.vstack([A[:1], A[:1]])
    y2 = np.array([1.0, -1.0])
    g2 = O.logistic_grad(A2, y2, np.zeros(d), lam, np.float64)
    assert np.allclose(g2, 0, atol=1e-16)
    xr = np.array([0.5, -2.0, 0.0])
    reg_only = O.logistic_grad(np.zeros((1, 3)), np.array([1.0]), xr, 0.3, np.float64)
    assert np.allclose(reg_only, 2 * 0.3 * xr / (1 + xr ** 2) ** 2, rtol=1e-15)
    # loss at zero is log 2
    assert abs(O.logistic_loss(A, yl, np.zeros(d), lam) - math.log(2)) < 1e-15


# ------------------------------------------------------------ reductions
def _wl(dtype=np.float64):
    wl = W.tiny(seed=1, T=30)
    return wl, wl.shards()


def _grads(shards, x, lam, dtype):
    return np.stack([O.logistic_grad(A, y, x, lam, dtype) for A, y in shards])


def test_identity_compressors_give_gradient_descent():
    # Eq. (2) with M = identity: x^{t+1} = x^t - gamma * mean_i grad f_i(x^t); exact in float64.
    wl, shards = _wl()
    o = O.AdaCGDOracle(n=wl.n, d=wl.d, gamma=wl.gamma, worker_levels=[(T, wl.d)], zeta_worker=0.0,
                       shards=shards, lam=wl.lam, dtype=np.float64)
    o.init(np.zeros(wl.d))
    x = np.zeros(wl.d)
    for t in range(30):
        g = _grads(shards, x, o.lam, np.float64)
        acc = np.zeros(wl.d)
        for i in range(wl.n):
            acc += g[i]
        x = x - o.gamma * (acc / wl.n)
        o.step()
        assert np.allclose(o.x, x, rtol=0, atol=1e-13)
    assert np.abs(o.x).max() > 1e-2


def test_single_level_zero_trigger_is_ef21():
    # zeta = 0, one Top-K level  ->  g_i <- g_i + TopK(grad - g_i)  (Eq. (7) inside Eq. (2)).
    wl, shards = _wl()
    K = 5
    o = O.AdaCGDOracle(n=wl.n, d=wl.d, gamma=wl.gamma, worker_levels=[(T, K)], zeta_worker=0.0,
                       shards=shards, lam=wl.lam, dtype=np.float64)
    o.init(np.zeros(wl.d), init_mode=O.INIT_ZERO)
    x = np.zeros(wl.d)
    gi = np.zeros((wl.n, wl.d))
    for t in range(30):
        x = x - o.gamma * gi.mean(0)
        for i, (A, y) in enumerate(shards):
            v = O.logistic_grad(A, y, x, o.lam, np.float64) - gi[i]
            keep = np.lexsort((np.arange(wl.d), -np.abs(v)))[:K]
            gi[i, keep] += v[keep]
        o.step()
        assert np.allclose(o.gi, gi, rtol=0, atol=1e-13)
        assert np.allclose(o.x, x, rtol=0, atol=1e-13)
        assert np.allclose(o.gt, o.gi.mean(0), rtol=0, atol=1e-13)      # Algorithm 1, aggregation line


@pytest.mark.parametrize("K", [3, 100])       # K = d makes C the identity: LAG
def test_single_level_with_trigger_is_clag(K):
    # m = 1: Eq. (8) -- send iff ||x - h||^2 > zeta ||x - y||^2.
    wl, shards = _wl()
    zeta = 4.0
    o = O.AdaCGDOracle(n=wl.n, d=wl.d, gamma=wl.gamma, worker_levels=[(T, K)], zeta_worker=zeta,
                       shards=shards, lam=wl.lam, dtype=np.float64)
    o.init(np.zeros(wl.d))
    x = np.zeros(wl.d)
    prev = _grads(shards, x, o.lam, np.float64)
    gi = prev.copy()
    sent = 0
    for t in range(30):
        x = x - o.gamma * gi.mean(0)
        new = _grads(shards, x, o.lam, np.float64)
        for i in range(wl.n):
            if np.sum((new[i] - gi[i]) ** 2) > zeta * np.sum((new[i] - prev[i]) ** 2):
                v = new[i] - gi[i]
                keep = np.lexsort((np.arange(wl.d), -np.abs(v)))[:K]
                gi[i, keep] += v[keep]
                sent += 1
        prev = new
        o.step()
        assert np.allclose(o.gi, gi, rtol=0, atol=1e-13)
        assert np.allclose(o.x, x, rtol=0, atol=1e-13)
    assert 0 < sent < 30 * wl.n          # both branches occurred
    assert o.level_hist_w[1] == sent and o.level_hist_w[0] == 30 * wl.n - sent


def test_zero_trigger_uses_last_level():
    # zeta = 0: every earlier trigger needs zero realised error, so the method is EF21 with C^m.
    wl, shards = _wl()
    lv = [(T, 1), (T, 5), (T, 25)]
    a = O.AdaCGDOracle(n=wl.n, d=wl.d, gamma=wl.gamma, worker_levels=lv, zeta_worker=0.0, shards=shards,
                       lam=wl.lam, dtype=np.float64)
    b = O.AdaCGDOracle(n=wl.n, d=wl.d, gamma=wl.gamma, worker_levels=lv[-1:], zeta_worker=0.0, shards=shards,
                       lam=wl.lam, dtype=np.float64)
    a.init(np.zeros(wl.d), init_mode=O.INIT_ZERO)
    b.init(np.zeros(wl.d), init_mode=O.INIT_ZERO)
    for t in range(20):
        a.step()
        b.step()
        assert np.array_equal(a.x, b.x) and np.array_equal(a.gi, b.gi)


# ------------------------------------------------------------ invariants
@pytest.mark.parametrize("dtype,tol", [(np.float64, 1e-13), (np.float32, 2e-6)])
def test_aggregate_is_mean_of_estimators_and_master_forms(dtype, tol):
    wl, shards = _wl()
    o = O.AdaCGDOracle(n=wl.n, d=wl.d, gamma=wl.gamma, worker_levels=wl.worker_levels, zeta_worker=1.0,
                       master_levels=wl.master_levels, zeta_master=0.0, shards=shards, lam=wl.lam, dtype=dtype)
    o.init(np.zeros(wl.d))
    seen = set()
    for t in range(60):
        g_before, gt_before = o.g.copy(), o.gt.copy()
        res, rm = o.step()
        seen.update(r.level for r in res)
        assert np.allclose(o.gt, o.gi.astype(np.float64).mean(0), rtol=0, atol=tol)   # Algorithm 1
        assert np.array_equal(o.gt_prev, gt_before)
        # master step in EF21 form: g <- g + TopK(g~ - g)
        vm = (o.gt - g_before).astype(dtype)
        keep = np.sort(np.lexsort((np.arange(wl.d), -np.abs(vm)))[:25])
        if rm.level == 1:
            assert rm.msg_idx.tolist() == keep.tolist()
            exp = g_before.copy()
            exp[keep] = (g_before[keep] + vm[keep]).astype(dtype)
            assert np.array_equal(o.g, exp)
        else:
            assert rm.level == 0 and rm.S == 0.0
    assert len(seen) >= 3            # the cascade visited several branches


def test_identity_master_equals_unidirectional():
    wl, shards = _wl()
    kw = dict(n=wl.n, d=wl.d, gamma=wl.gamma, worker_levels=wl.worker_levels, zeta_worker=1.0, shards=shards,
              lam=wl.lam, dtype=np.float32)
    a = O.AdaCGDOracle(**kw)
    b = O.AdaCGDOracle(master_levels=[(T, wl.d)], zeta_master=0.0, **kw)
    a.init(np.zeros(wl.d))
    b.init(np.zeros(wl.d))
    for t in range(25):
        a.step()
        b.step()
        assert np.array_equal(a.g, a.gt)
        # h + (x - h) is x only up to one rounding of the difference and one of the sum
        assert np.allclose(b.g, b.gt, rtol=3e-7, atol=1e-9)
        assert np.allclose(a.x, b.x, rtol=0, atol=1e-6)


def test_previous_gradient_advances_on_skip():
    # Algorithm 2: y is grad f_i(x^t), the previous iterate's gradient, whatever branch was taken.
    wl, shards = _wl()
    o = O.AdaCGDOracle(n=wl.n, d=wl.d, gamma=wl.gamma, worker_levels=[(T, 5)], zeta_worker=1e6, shards=shards,
                       lam=wl.lam, dtype=np.float32)
    o.init(np.zeros(wl.d))
    res, _ = o.step()
    assert all(r.level == 0 for r in res)
    assert np.array_equal(o.y, _grads(shards, o.x, o.lam, np.float32))


def test_counters():
    lv = [(T, 4), (O.QUANT, 4), (T, 64)]
    d = 100
    idb = 2
    assert O.AdaCGDOracle.message_bits(0, lv, d) == idb
    assert O.AdaCGDOracle.message_bits(1, lv, d) == idb + 4 * (32 + 7)
    assert O.AdaCGDOracle.message_bits(2, lv, d) == idb + d * 4 + 32
    assert [O.AdaCGDOracle.message_values(j, lv, d) for j in range(4)] == [0, 4, d, 64]


def test_quantiser_level_inside_cascade_is_ef21_with_dense_message():
    rng = np.random.default_rng(41)
    d = 64
    h = rng.standard_normal(d).astype(np.float32)
    x = (h + rng.standard_normal(d)).astype(np.float32)
    y = (x + 0.01 * rng.standard_normal(d)).astype(np.float32)
    r = O.adacgd_compress(h, y, x, [(T, 1), (O.QUANT, 8)], 1.0, seed=5, node=2, step=3)
    assert r.level == 2
    v = (x - h).astype(np.float32)
    c, codes, scale = O.quantize(v, 8, O.dither_uniforms(d, 5, 2, 3))
    assert np.array_equal(r.h_new, (h + c).astype(np.float32))
    assert r.err[1] == O.sum_sq_diff(v, c)


# ------------------------------------------------------------ general triggers (Section 4.2, Lemma 2)
def test_triggers_default_is_the_adacgd_definition():
    rng = np.random.default_rng(5)
    levels = [(T, 2), (T, 8), (O.QUANT, 4), (T, 40)]
    for zeta in (0.0, 0.3, 1.0, 7.0):
        for _ in range(20):
            h, y, x = (rng.standard_normal(64).astype(np.float32) for _ in range(3))
            a = O.adacgd_compress(h, y, x, levels, zeta, seed=3, node=1, step=2)
            b = O.adacgd_compress(h, y, x, levels, 123.0, seed=3, node=1, step=2, triggers=[(zeta, 0.0)] * 4)
            assert a.level == b.level and np.array_equal(a.h_new, b.h_new) and a.err == b.err


def test_trigger_decision_table_with_both_terms():
    # v = (4,3,2,1): S = 30, Top-1/2/3 errors 14, 5, 1; D = 4.
    v = np.array([4.0, -3, 2, -1])
    levels = [(T, 1), (T, 2), (T, 3), (T, 4)]

    def level(trig):
        return O.adacgd_compress(np.zeros(4), None, None, levels, 0.0, D_given=4.0, v_given=v, triggers=trig).level

    assert level([(0, 0)] * 4) == 4                                   # nothing is accepted: last level
    assert level([(7.5, 0), (0, 0), (0, 0), (0, 0)]) == 0             # 30 <= 7.5 * 4
    assert level([(7.4, 0), (3.5, 0), (0, 0), (0, 0)]) == 1           # 30 > 29.6, 14 <= 14
    assert level([(0, 0.99), (0, 0.4), (0, 0.2), (0, 0)]) == 2        # 30 > 29.7, 14 > 12, 5 <= 6
    assert level([(0, 1.0), (0, 0), (0, 0), (0, 0)]) == 0             # eta_0 = 1 always keeps h
    assert level([(0, 0), (1.25, 0.3), (0, 0), (0, 0)]) == 1          # 14 <= 5 + 9
    assert level([(0, 0), (1.2, 0.3), (1.25, 0), (0, 0)]) == 2        # 14 > 13.8, 5 <= 5
    assert level([(0, 0), (0, 0), (0, 0), (0.25, 0)]) == 3            # 1 <= 1
    assert level([(0, 0), (0, 0), (0, 0), (0.2, 0.005)]) == 4         # 1 > 0.8 + 0.15
    assert level([(0, 0), (0, 0), (0, 0), (0.2, 0.02)]) == 3          # 1 <= 0.8 + 0.6


def test_relative_error_triggers_pick_the_smallest_sufficient_K():
    """zeta_j = 0, eta_j = eta: the cascade accepts the first Top-K level whose realised error is at
    most eta ||v||^2.  Recomputed here from the sorted squares: the error of Top-K is the energy
    of the d - K smallest magnitudes."""
    rng = np.random.default_rng(11)
    Ks = [1, 3, 10, 30, 100, 300]
    levels = [(T, k) for k in Ks]
    seen = set()
    for trial in range(60):
        d = 300
        v = (rng.standard_normal(d) * np.exp(rng.uniform(0, 4) * rng.standard_normal(d))).astype(np.float64)
        eta = float(rng.choice([0.5, 0.1, 0.01, 1e-4]))
        r = O.adacgd_compress(np.zeros(d), None, None, levels, 0.0, D_given=1.0, v_given=v,
                              triggers=[(0.0, eta)] * len(Ks))
        sq = np.sort(v * v)                      # ascending
        tail = np.concatenate([[0.0], np.cumsum(sq)])          # tail[q] = energy of the q smallest
        want = len(Ks)
        for j, k in enumerate(Ks[:-1], start=1):
            if tail[d - k] <= eta * tail[d]:
                want = j
                break
        if min(r.margins) > 1e-9:
            assert r.level == want, (trial, eta)
        seen.add(r.level)
        # contractive by construction with alpha = 1 - eta (last level is the identity here)
        assert O.sum_sq_diff(r.h_new, v) <= eta * r.S * (1 + 1e-12)
    assert len(seen) >= 4


def test_per_level_zeta_is_first_condition_that_holds():
    rng = np.random.default_rng(12)
    levels = [(T, 1), (T, 4), (O.QUANT, 3), (T, 32), (T, 64)]
    hist = np.zeros(6, dtype=int)
    for trial in range(200):
        h, y, x = (rng.standard_normal(64).astype(np.float32) for _ in range(3))
        y = (x + rng.uniform(0.05, 1.5) * (y - x)).astype(np.float32)
        trig = [(float(rng.uniform(0, 2)), float(rng.uniform(0, 0.6))) for _ in levels]
        r = O.adacgd_compress(h, y, x, levels, 0.0, seed=1, node=0, step=trial, triggers=trig)
        lhs = [r.S] + r.err[:-1]
        rhs = [float(np.float32(z)) * r.D + float(np.float32(e)) * r.S for z, e in trig]
        first = next((j for j in range(5) if lhs[j] <= rhs[j]), 5)
        assert r.level == first
        hist[r.level] += 1
    assert (hist > 0).sum() >= 5


def test_compressed_start_is_topk_of_the_first_gradients():
    """INIT_COMPRESSED: g~_i^0 = C_m(grad f_i(x^0)) (the CLAG / EF21 start, Section 2.3), here against a
    sort of (|value|, index) pairs, compared as bit patterns: a selected coordinate keeps the gradient's
    value exactly, the sign of a selected zero included.  The run that follows with zeta = 0 and one level
    is EF21 from that start."""
    rng = np.random.default_rng(21)
    n, d, K = 3, 40, 7
    g0 = rng.standard_normal((n, d)).astype(np.float32)
    g0[0, ::2] = 0.0
    g0[0, 1] = -0.0
    g0[1, :] = 0.0                   # fewer non-zeros than K: zeros are selected by ascending index ...
    g0[1, [1, 3]] = -0.0             # ... and these two are among them
    g0[1, [20, 30, 35]] = (1.5, -2.5, 0.5)
    orc = O.AdaCGDOracle(n=n, d=d, gamma=0.1, worker_levels=[(T, 2), (T, K)], zeta_worker=0.0)
    orc.init(np.zeros(d, dtype=np.float32), g0, O.INIT_COMPRESSED)
    for i in range(n):
        order = sorted(range(d), key=lambda l: (-abs(float(g0[i, l])), l))[:K]
        want = np.zeros(d, dtype=np.float32)
        want[order] = g0[i, order]
        assert np.array_equal(orc.gi[i].view(np.uint32), want.view(np.uint32))
    assert orc.gi[1].view(np.uint32)[[0, 1, 2, 3]].tolist() == [0, 0x80000000, 0, 0x80000000]
    assert np.allclose(orc.gt, orc.gi.astype(np.float64).mean(0), rtol=1e-7, atol=0)
    h = orc.gi.copy()
    g1 = (g0 + 0.1 * rng.standard_normal((n, d))).astype(np.float32)
    orc.step(grads=g1)
    for i in range(n):
        v = g1[i] - h[i]
        order = sorted(range(d), key=lambda l: (-abs(float(v[l])), l))[:K]
        want = h[i].copy()
        want[order] = h[i][order] + v[order]
        assert np.array_equal(orc.gi[i].view(np.uint32), want.view(np.uint32))


def test_stored_trajectory_is_reproduced():
    """tests/golden/trajectory_tiny_external.txt (written by make_trajectory_golden.py from the oracle
    alone) still comes out of the oracle: level choices, supports and every state vector, bit for bit."""
    import importlib.util
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_trajectory_golden", os.path.join(here, "make_trajectory_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = open(os.path.join(here, "trajectory_tiny_external.txt")).read().splitlines()
    assert mod.lines() == stored
    levels = {int(v) for line in stored[1:] for v in line.split("|")[1].split()}
    assert levels == {0, 1, 2, 3, 4}                      # the stored run visits every branch of the cascade
