"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element,
on the same seeded inputs.  Compression step: chosen level, selected coordinates,
message values and updated estimators are compared bit for bit; the fp64 reductions
(||x-h||^2, ||x-y||^2, err_j) to 1e-12 relative (both sides accumulate in fp64 or
wider, only the summation order differs).  Iterates and gradients: 1e-5 relative."""
import contextlib

import numpy as np
import pytest

from oracle import adacgd_oracle as O
from paper_2211_00188_amd import workloads as W

pytestmark = pytest.mark.gpu

RED_RTOL = 1e-12      # fp64 reductions
TRAJ_RTOL = 1e-5      # iterates, gradients (fp32 storage)


def _eng():
    from paper_2211_00188_amd import engine as E
    return E


def _cuda(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


def by_alpha(levels, d):
    """A mixed level set in the order of the AdaCGD definition (contraction parameter ascending,
    stable), with the oracle's contraction parameters."""
    return sorted(levels, key=lambda lv: O.level_alpha(lv, d))


ELT_FLOOR_UNITS = 16      # absolute floor of the element-wise check, in units of 2^-24 max|b|


def assert_close_rel(a, b, rtol, what):
    """Max-norm check |a - b|_inf <= rtol |b|_inf, and element by element
    |a_l - b_l| <= rtol |b_l| + floor with floor = ELT_FLOOR_UNITS 2^-24 |b|_inf: coordinates far below
    the largest one inherit absolute errors of that size through the coupling of the coordinates
    (a gradient coordinate depends on every coordinate of the iterate), so a purely relative bound
    cannot hold for them; the floor is a few units in the last place of the largest element."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    scale = max(np.abs(b).max(), 1e-300)
    assert np.abs(a - b).max() <= rtol * scale, (what, np.abs(a - b).max() / scale)
    excess = np.abs(a - b) - (rtol * np.abs(b) + ELT_FLOOR_UNITS * 2.0 ** -24 * scale)
    assert excess.max() <= 0, (what, "element-wise", int(np.argmax(excess)), float(excess.max() / scale))


def min_margin(res):
    ms = [m for r in res for m in r.margins]
    return min(ms) if ms else 1.0


class NearTie(Exception):
    """A trigger comparison of this step is within 1e-12 (relative) of equality.  The two sides of the
    comparison are fp64 sums whose order of summation differs between the oracle and the kernels, so
    either decision is correct there, and the two runs may continue on different branches."""


NEAR_TIE_RUNS = []          # runs whose comparison was cut short at a near tie, over the whole session
MAX_NEAR_TIE_RUNS = 3       # expected: none


@contextlib.contextmanager
def until_near_tie(tag):
    """Wraps the comparison loop of one engine / oracle pair.  A near tie ends the comparison of that
    pair at the step where it occurs (everything before it has been compared); the test is never
    skipped, and the number of such cuts is bounded over the session."""
    try:
        yield
    except NearTie as e:
        NEAR_TIE_RUNS.append((tag, str(e)))
        print("near tie, comparison of this run ends here:", tag, e)
        assert len(NEAR_TIE_RUNS) <= MAX_NEAR_TIE_RUNS, NEAR_TIE_RUNS


def compare_step(eng, orc, res, rm, tag, check_master=True):
    """Bit-exact comparison of one step's compression outputs.  Raises NearTie (after the reductions
    have been compared) if a trigger comparison of the step is too close to equality to be decided
    by sums that differ in their order of summation."""
    E = _eng()
    n = orc.n
    lev = eng.state(E.F_LEVEL)
    S, D, err = eng.state(E.F_SQNORM), eng.state(E.F_D), eng.state(E.F_ERR)
    near_tie = min_margin(res + ([rm] if (check_master and rm is not None) else [])) < 1e-12
    for i, r in enumerate(res):
        assert abs(S[i] - r.S) <= RED_RTOL * max(r.S, 1e-300), (tag, i, "S")
        assert abs(D[i] - r.D) <= RED_RTOL * max(r.D, 1e-300), (tag, i, "D")
        if r.level == 0 and not near_tie:
            # the cascade stops at its first condition: a skipping node's level errors are not evaluated
            assert np.isnan(err[i]).all(), (tag, i, "err of a skipped node")
            continue
        for j, e in enumerate(r.err):
            if near_tie and np.isnan(err[i, j]):
                continue
            assert abs(err[i, j] - e) <= RED_RTOL * max(e, r.S * 1e-6, 1e-300), (tag, i, j, "err", err[i, j], e)
    if near_tie:
        raise NearTie(repr(tag))
    assert lev.tolist() == [r.level for r in res], (tag, "levels")
    msgs = eng.messages()
    for i, r in enumerate(res):
        assert np.array_equal(msgs[i][0], r.msg_idx), (tag, i, "msg idx")
        assert np.array_equal(bits(msgs[i][1]), bits(r.msg_val)), (tag, i, "msg val")
    gi = eng.state(E.F_GI)
    assert np.array_equal(bits(gi), bits(orc.gi)), (tag, "g_i")
    assert np.array_equal(bits(eng.state(E.F_GTILDE)), bits(orc.gt)), (tag, "g~")
    assert np.array_equal(bits(eng.state(E.F_GTILDE_PREV)), bits(orc.gt_prev)), (tag, "g~ prev")
    if check_master:
        assert np.array_equal(bits(eng.state(E.F_G)), bits(orc.g)), (tag, "g")
        if rm is not None:
            assert int(eng.state(E.F_M_LEVEL)[0]) == rm.level
            assert np.array_equal(eng.state(E.F_M_MSG_IDX), rm.msg_idx)
            assert np.array_equal(bits(eng.state(E.F_M_MSG_VAL)), bits(rm.msg_val))
    assert np.array_equal(bits(eng.state(E.F_X)), bits(orc.x)), (tag, "x")
    # G = (1/n) sum ||x_i - g~_i||^2 after the update: the realised error of what each worker applied
    want = np.mean([r.S if r.level == 0 else r.err[r.level - 1] for r in res])
    got = float(eng.state(E.F_ESTIMATOR_ERR)[0])
    assert abs(got - want) <= RED_RTOL * max(want, 1e-300), (tag, "G", got, want)


def make_vectors(rng, n, d, kind):
    if kind == "normal":
        return rng.standard_normal((n, d)).astype(np.float32)
    if kind == "ties":        # few distinct magnitudes: every threshold falls inside a run of ties
        return (rng.integers(-3, 4, size=(n, d)) * 0.5).astype(np.float32)
    if kind == "heavy":
        return (rng.standard_t(3, size=(n, d)) * np.exp(rng.standard_normal((n, 1)))).astype(np.float32)
    if kind == "sparse":      # fewer non-zeros than K for the larger levels; signed zeros
        v = rng.standard_normal((n, d)).astype(np.float32)
        v[rng.random((n, d)) < 0.97] = 0.0
        v[rng.random((n, d)) < 0.3] *= -1.0
        return v
    if kind == "denormal":
        return (rng.standard_normal((n, d)) * 1e-41).astype(np.float32)
    if kind == "const":
        return np.full((n, d), -2.5, dtype=np.float32)
    raise ValueError(kind)


SHAPES = [
    (3, 3 * 8192 + 516),     # several tiles + ragged tail, 16-byte vector path
    (2, 2 * 8192 + 517),     # d % 4 != 0: scalar path
    (5, 1000),               # one partial tile
    (1, 1),                  # degenerate
    (2, 8192),               # exactly one tile
]


@pytest.mark.parametrize("kind", ["normal", "ties", "heavy", "sparse", "denormal", "const"])
@pytest.mark.parametrize("n,d,general", [(n, d, False) for n, d in SHAPES] +
                         [(5, 1000, True), (1, 1, True), (3, 4096, False), (2, 4095, True)])
def test_compression_step_bit_exact_external_gradients(n, d, kind, general):
    """`general`: short vectors through the general two-pass kernels instead of the one-block kernel."""
    E = _eng()
    rng = np.random.default_rng(1000 + d + len(kind))
    Ks = sorted({max(1, min(d, k)) for k in (1, 7, d // 50, d // 8, d // 2, d)})
    wl = [(O.TOPK, k) for k in Ks]
    ml = [(O.TOPK, max(1, d // 10))]
    steps = 4
    grads = [make_vectors(rng, n, d, kind) for _ in range(steps + 1)]
    for t in range(1, steps + 1):      # consecutive gradients differ by a small, varying amount
        grads[t] = (grads[t - 1] + grads[t] * np.float32(10.0 ** rng.uniform(-2, 0))).astype(np.float32)
    x0 = rng.standard_normal(d).astype(np.float32)
    for zeta in (0.0, 0.6, 3.0):
        orc = O.AdaCGDOracle(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=zeta, master_levels=ml,
                             zeta_master=0.0)
        orc.init(x0, grads[0], O.INIT_ZERO if zeta == 0.6 else O.INIT_FULLGRAD)
        eng = E.AdaCGD(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=zeta, master_levels=ml,
                       zeta_master=0.0, grad_mode=E.GRAD_EXTERNAL,
                       init_mode=E.INIT_ZERO if zeta == 0.6 else E.INIT_FULLGRAD, x0=_cuda(x0),
                       grad0=_cuda(grads[0]), flags=E.FLAG_TWO_PASS if general else 0)
        assert np.array_equal(bits(eng.state(E.F_GTILDE)), bits(orc.gt))
        with until_near_tie((n, d, kind, zeta)):
            for t in range(1, steps + 1):
                res, rm = orc.step(grads=grads[t])
                eng.step(_cuda(grads[t]))
                compare_step(eng, orc, res, rm, (n, d, kind, zeta, t))
                assert np.array_equal(bits(eng.state(E.F_PREV_GRAD)), bits(grads[t]))
            hist = eng.state(E.F_LEVEL_HIST)
            assert hist.tolist() == orc.level_hist_w.tolist()
        eng.close()


def test_retained_external_gradient_pointer_matches_copy():
    E = _eng()
    rng = np.random.default_rng(5)
    n, d = 3, 20000
    wl = [(O.TOPK, 10), (O.TOPK, 500)]
    grads = [_cuda(rng.standard_normal((n, d)).astype(np.float32)) for _ in range(4)]
    x0 = _cuda(np.zeros(d, dtype=np.float32))
    out = []
    for flags in (0, E.FLAG_RETAIN_EXT):
        eng = E.AdaCGD(n=n, d=d, worker_levels=wl, zeta_worker=0.5, grad_mode=E.GRAD_EXTERNAL, x0=x0,
                       grad0=grads[0], flags=flags)
        for t in range(1, 4):
            eng.step(grads[t])
        out.append((eng.state(E.F_GI), eng.state(E.F_X), eng.state(E.F_PREV_GRAD)))
        eng.close()
    for a, b in zip(*out):
        assert np.array_equal(bits(a), bits(b))


@pytest.mark.parametrize("n,d", [(4, 3 * 8192 + 40), (3, 5003), (6, 3001)])
def test_difference_mode_with_quantiser_levels_bit_exact(n, d):
    """Caller-supplied difference vectors and trigger right-hand sides; mixed Top-K and
    b-bit levels ordered by contraction parameter; every branch of the cascade occurs."""
    E = _eng()
    wk = W.kernel_stress(seed=3, n=n, d=d)
    wk.worker_levels = by_alpha(wk.worker_levels, d)
    seed = 0x1234ABCD5678
    orc = O.AdaCGDOracle(n=n, d=d, gamma=0.1, worker_levels=wk.worker_levels, zeta_worker=1.0,
                         master_levels=wk.master_levels, zeta_master=0.0, seed=seed)
    x0 = np.zeros(d, dtype=np.float32)
    orc.init(x0, None, O.INIT_ZERO)
    eng = E.AdaCGD(n=n, d=d, gamma=0.1, worker_levels=wk.worker_levels, zeta_worker=1.0,
                   master_levels=wk.master_levels, zeta_master=0.0, grad_mode=E.DIFF_EXTERNAL,
                   init_mode=E.INIT_ZERO, x0=_cuda(x0), seed=seed)
    seen = set()
    with until_near_tie(("diff", n, d)):
        for t in range(8):
            v, D = W.kernel_stress_diffs(wk, t)
            res, rm = orc.step(diffs=v, D=D)
            eng.step(_cuda(v), _cuda(D))
            seen.update(r.level for r in res)
            compare_step(eng, orc, res, rm, ("diff", n, d, t))
            for i, r in enumerate(res):
                if r.dense is not None:
                    codes = eng.state(E.F_QCODES)[i]
                    assert np.array_equal(codes.astype(np.int32), r.codes), ("codes", t, i)
                    assert eng.state(E.F_QSCALE)[i] == np.float32(r.scale)
        kinds = {wk.worker_levels[j - 1][0] for j in seen if j > 0}
        assert 0 in seen and kinds == {O.TOPK, O.QUANT}, seen
    eng.close()


def _logistic_engine(wl, zeta=None, x0=None, **kw):
    E = _eng()
    A, labels = _cuda(wl.A), _cuda(wl.labels)
    x0 = _cuda(np.zeros(wl.d, dtype=np.float32) if x0 is None else x0)
    return E.AdaCGD(n=wl.n, d=wl.d, gamma=wl.gamma, lam=wl.lam, worker_levels=wl.worker_levels,
                    zeta_worker=wl.zeta_worker if zeta is None else zeta, master_levels=wl.master_levels,
                    zeta_master=wl.zeta_master, grad_mode=E.GRAD_LOGISTIC, A=A, labels=labels,
                    shard_offsets=wl.shard_offsets, x0=x0, **kw)


def _logistic_oracle(wl, zeta=None, seed=0, x0=None):
    orc = O.AdaCGDOracle(n=wl.n, d=wl.d, gamma=wl.gamma, worker_levels=wl.worker_levels,
                         zeta_worker=wl.zeta_worker if zeta is None else zeta, master_levels=wl.master_levels,
                         zeta_master=wl.zeta_master, shards=wl.shards(), lam=wl.lam, seed=seed)
    orc.init(np.zeros(wl.d, dtype=np.float32) if x0 is None else x0)
    return orc


def run_trajectory(wl, T, zeta=None, check_every=1, seed=0, x0=None):
    E = _eng()
    orc = _logistic_oracle(wl, zeta, seed, x0)
    eng = _logistic_engine(wl, zeta, x0, seed=seed)
    assert_close_rel(eng.state(E.F_GRAD), orc.y, TRAJ_RTOL, "grad0")
    levels_equal = 0
    for t in range(T):
        res, rm = orc.step()
        eng.step()
        if (t + 1) % check_every == 0 or t == T - 1:
            assert_close_rel(eng.state(E.F_X), orc.x, TRAJ_RTOL, ("x", t))
            assert_close_rel(eng.state(E.F_GRAD), orc.y, TRAJ_RTOL, ("grad", t))
            assert_close_rel(eng.state(E.F_G), orc.g, TRAJ_RTOL, ("g", t))
            levels_equal += int(eng.state(E.F_LEVEL).tolist() == [r.level for r in res])
    hist = eng.state(E.F_LEVEL_HIST).astype(np.int64)
    eng.close()
    return orc, hist, levels_equal


@pytest.mark.parametrize("zeta", [0.0, 1.0, 16.0])
def test_trajectory_tiny_logistic(zeta):
    wl = W.tiny()
    orc, hist, _ = run_trajectory(wl, wl.T, zeta=zeta)
    assert hist.tolist() == orc.level_hist_w.tolist()
    assert hist.sum() == wl.T * wl.n


def test_trajectory_sparse_logreg():
    """The full sparse-logreg configuration (T = 1000, 20000 level decisions): iterate, gradients and g
    within 1e-5 at every step.  The two sides' gradients agree to about one fp32 unit, not bit for bit
    (the order of the fp64 summation differs), so a trigger comparison that close to equality may fall
    either way.  Every decision that differs must be explained that way: the two sides of the
    comparison, as norms, are 1-Lipschitz in the vectors they are formed from (||v - TopK(v)|| is the
    distance of v to the K-sparse vectors), so a decision can differ only if the oracle's gap
    | sqrt(lhs) - sqrt(zeta D) | is at most what the measured difference of the inputs (gradient,
    previous gradient, estimator) allows, plus the rounding of the two subtractions."""
    E = _eng()
    wl = W.sparse_logreg()                 # the full configuration: T = 1000
    orc = _logistic_oracle(wl)
    eng = _logistic_engine(wl)
    zeta = float(np.float32(wl.zeta_worker))
    assert_close_rel(eng.state(E.F_GRAD), orc.y, TRAJ_RTOL, "grad0")
    nrm = lambda a: float(np.sqrt(np.sum(np.asarray(a, dtype=np.float64) ** 2)))
    flips = []
    for t in range(wl.T):
        y_o, y_e = orc.y.copy(), eng.state(E.F_GRAD)
        h_o, h_e = orc.gi.copy(), eng.state(E.F_GI)
        res, rm = orc.step()
        eng.step()
        x_e = eng.state(E.F_GRAD)
        assert_close_rel(eng.state(E.F_X), orc.x, TRAJ_RTOL, ("x", t))
        assert_close_rel(x_e, orc.y, TRAJ_RTOL, ("grad", t))
        assert_close_rel(eng.state(E.F_G), orc.g, TRAJ_RTOL, ("g", t))
        lev = eng.state(E.F_LEVEL)
        for i, r in enumerate(res):
            if lev[i] == r.level:
                continue
            pos = min(int(lev[i]), r.level)          # cascade position that one side accepted and the other did not
            lhs = r.S if pos == 0 else r.err[pos - 1]
            dx, dy, dh = nrm(x_e[i] - orc.y[i]), nrm(y_e[i] - y_o[i]), nrm(h_e[i] - h_o[i])
            gap = abs(np.sqrt(lhs) - np.sqrt(zeta * r.D))
            allowed = (dx + dh) + np.sqrt(zeta) * (dx + dy) + 2.0 ** -23 * (np.sqrt(r.S) + np.sqrt(zeta * r.D))
            assert gap <= allowed, (t, i, int(lev[i]), r.level, gap, allowed)
            flips.append((t, i, int(lev[i]), r.level, gap / max(np.sqrt(lhs), 1e-300)))
    hist = eng.state(E.F_LEVEL_HIST).astype(np.int64)
    eng.close()
    print("decisions that differ (step, worker, engine level, oracle level, relative gap):", flips)
    assert len(flips) <= 10, flips            # of 20000; one when first measured
    assert (hist > 0).sum() >= 3              # the cascade used several levels


def test_trajectory_federated_reduced():
    wl = W.federated(n=24, d=8192 + 512, N=32, T=20)
    wl.worker_levels = by_alpha(wl.worker_levels, wl.d)
    orc, hist, _ = run_trajectory(wl, wl.T, check_every=1, seed=77)
    assert hist.tolist() == orc.level_hist_w.tolist()


def test_trajectory_odd_dimension_uneven_shards():
    wl = W.tiny(seed=9, n=3, d=101, N=50, T=40)
    wl.shard_offsets = np.array([0, 20, 90, 150], dtype=np.int64)
    # At x = 0 every margin term is -y_l / (2 N_i): with N_i = 20 the exact gradient often lies
    # midway between two fp32 numbers and the fp64 summation order decides the rounding; a random
    # starting point removes that structure.
    x0 = (0.1 * np.random.default_rng(9).standard_normal(wl.d)).astype(np.float32)
    orc, hist, _ = run_trajectory(wl, wl.T, x0=x0)
    assert hist.tolist() == orc.level_hist_w.tolist()


def test_communication_counters():
    E = _eng()
    wl = W.tiny(T=30)
    orc = _logistic_oracle(wl)
    eng = _logistic_engine(wl)
    up_v = up_b = dn_v = dn_b = 0
    for t in range(30):
        res, rm = orc.step()
        eng.step()
        for r in res:
            up_v += O.AdaCGDOracle.message_values(r.level, orc.wl, wl.d)
            up_b += O.AdaCGDOracle.message_bits(r.level, orc.wl, wl.d)
        dn_v += wl.n * O.AdaCGDOracle.message_values(rm.level, orc.ml, wl.d)
        dn_b += wl.n * O.AdaCGDOracle.message_bits(rm.level, orc.ml, wl.d)
    assert eng.state(E.F_COMM).tolist() == [up_v, up_b, dn_v, dn_b]
    assert int(eng.state(E.F_STEP)[0]) == 30
    eng.close()


@pytest.mark.parametrize("n,d,N", [(4, 100, 64), (3, 101, 50), (5, 8192 + 12, 7), (2, 300, 2500)])
def test_gradient_kernel_matches_oracle(n, d, N):
    """grad f_i(x) of the logistic objective with the nonconvex regulariser at several
    points, through init (which evaluates it at x0).  Both sides accumulate in fp64 and
    round once to fp32: values agree to one fp32 unit in the last place."""
    E = _eng()
    wl = W.tiny(seed=21, n=n, d=d, N=N)
    rng = np.random.default_rng(d)
    for scale in (0.0, 0.05, 3.0):
        x0 = (scale * rng.standard_normal(d)).astype(np.float32)
        eng = _logistic_engine(wl, x0=x0)
        got = eng.state(E.F_GRAD)
        eng.close()
        ref = np.stack([O.logistic_grad(A, y, x0, np.float64(np.float32(wl.lam)), np.float32) for A, y in wl.shards()])
        ulp = np.spacing(np.abs(ref)).astype(np.float64)
        assert np.all(np.abs(got.astype(np.float64) - ref.astype(np.float64)) <= ulp)
        assert_close_rel(got, ref, TRAJ_RTOL, ("grad", n, d, N, scale))
        if scale > 0:
            assert np.mean(bits(got) != bits(ref)) < 0.01


def test_trajectory_with_oracle_gradients_is_bit_exact():
    """The whole step except the gradient kernel (iterate update, compression, level choice,
    aggregation, master compression) over many iterations, with the oracle's gradients fed
    to both sides: every vector must agree bit for bit at every step."""
    E = _eng()
    wl = W.sparse_logreg(n=10, N=400, T=150)
    orc = _logistic_oracle(wl)
    eng = E.AdaCGD(n=wl.n, d=wl.d, gamma=wl.gamma, worker_levels=wl.worker_levels, zeta_worker=wl.zeta_worker,
                   master_levels=wl.master_levels, zeta_master=wl.zeta_master, grad_mode=E.GRAD_EXTERNAL,
                   x0=_cuda(np.zeros(wl.d, dtype=np.float32)), grad0=_cuda(orc.y))
    for t in range(wl.T):
        res, rm = orc.step()
        eng.step(_cuda(orc.y))
        # 150 steps x 11 nodes of comparisons on this fixed input: none is within 1e-12 of equality
        assert min_margin(res + [rm]) >= 1e-12, t
        assert eng.state(E.F_LEVEL).tolist() == [r.level for r in res], t
        assert np.array_equal(bits(eng.state(E.F_X)), bits(orc.x)), t
        assert np.array_equal(bits(eng.state(E.F_G)), bits(orc.g)), t
        assert np.array_equal(bits(eng.state(E.F_GI)), bits(orc.gi)), t
        # the diagnostic G^t against its definition, from the vectors themselves
        direct = np.mean([O.sum_sq_diff(orc.y[i], orc.gi[i]) for i in range(wl.n)])
        # (h + C(v) is rounded to fp32: when everything is sent the realised error is 0 and the vectors
        # differ by that rounding only)
        floor = 1e-12 * np.mean([O.sum_squares(orc.y[i]) for i in range(wl.n)])
        assert abs(float(eng.state(E.F_ESTIMATOR_ERR)[0]) - direct) <= 1e-5 * direct + floor
    assert eng.state(E.F_LEVEL_HIST).tolist() == orc.level_hist_w.tolist()
    assert (orc.level_hist_w > 0).sum() >= 3
    eng.close()


def _sampled_row(t):
    """Row (of 32 rows of 256 coordinates) of tile t that the one-pass selection samples."""
    return ((t * 2654435761) & 0xFFFFFFFF) >> 27


@pytest.mark.parametrize("kind", ["normal", "heavy", "ties", "const", "sparse", "adversarial", "two_pass_flag"])
def test_long_vectors_one_pass_selection_bit_exact(kind):
    """Vectors long enough for the sampled one-pass selection (>= 128 tiles of 8192).  The
    'adversarial' input puts all large magnitudes exactly on the sampled rows, so the sampled
    cut-off estimate is far too high and the repair pass must produce the same exact result."""
    E = _eng()
    n, d = 2, 130 * 8192 + 1284
    rng = np.random.default_rng(77)
    wl = [(O.TOPK, 50), (O.TOPK, 3000), (O.TOPK, d // 20)]
    ml = [(O.TOPK, d // 100)]
    steps = 3
    base_kind = {"adversarial": "normal", "two_pass_flag": "normal"}.get(kind, kind)
    grads = [make_vectors(rng, n, d, base_kind) for _ in range(steps + 1)]
    if kind == "adversarial":
        for g in grads[1:]:
            for t in range((d + 8191) // 8192):
                lo = t * 8192 + _sampled_row(t) * 256
                g[:, lo:min(d, lo + 256)] *= np.float32(1000.0)
    for t in range(1, steps + 1):
        grads[t] = (grads[t - 1] * np.float32(0.5) + grads[t]).astype(np.float32)
    x0 = np.zeros(d, dtype=np.float32)
    zeta = 0.3
    orc = O.AdaCGDOracle(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=zeta, master_levels=ml, zeta_master=0.0)
    orc.init(x0, grads[0], O.INIT_FULLGRAD)
    eng = E.AdaCGD(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=zeta, master_levels=ml, zeta_master=0.0,
                   grad_mode=E.GRAD_EXTERNAL, x0=_cuda(x0), grad0=_cuda(grads[0]),
                   flags=E.FLAG_TWO_PASS if kind == "two_pass_flag" else 0)
    with until_near_tie(("long", kind)):
        for t in range(1, steps + 1):
            res, rm = orc.step(grads=grads[t])
            eng.step(_cuda(grads[t]))
            compare_step(eng, orc, res, rm, ("long", kind, t))
    repairs = eng.state(E.F_REPAIRS)
    if kind == "adversarial":
        assert repairs[0] > 0                    # the second scan did run
    if kind in ("normal", "heavy", "two_pass_flag"):
        assert repairs[0] == 0
    eng.close()


@pytest.mark.parametrize("mode", ["grad", "diff", "diff_quant", "diff_block_rank"])
def test_overlap_mode_gives_identical_results(mode):
    """Worker compression on the library's own stream, overlapped with the previous step's
    server work: every state vector and message must equal the single-stream run bit for bit,
    and the oracle, over enough steps for the two chains to interleave."""
    E = _eng()
    import torch
    n, d = 4, 140 * 8192 + 64
    rng = np.random.default_rng(123)
    wl = [(O.TOPK, 100), (O.TOPK, 5000), (O.TOPK, d // 25)]
    if mode == "diff_quant":       # dense quantised messages: their scales and codes are message tables too
        wl = by_alpha([(O.TOPK, 100), (O.QUANT, 2), (O.QUANT, 4), (O.TOPK, d // 25), (O.QUANT, 8)], d)
    any_order = 0
    if mode == "diff_block_rank":  # block-wise scales and Rank-K reconstructions are message tables as well
        wl = [(O.RANK, (1, 64)), (O.TOPK, 100), (O.RANK, (32, 64)), (O.QUANT_BLOCK, (2, 256)), (O.TOPK, d // 25),
              (O.QUANT_BLOCK, (8, 256))]
        any_order = E.FLAG_ANY_LEVEL_ORDER
    ml = [(O.TOPK, d // 100)]
    steps = 6
    x0 = _cuda(np.zeros(d, dtype=np.float32))
    if mode == "grad":
        host = [rng.standard_normal((n, d)).astype(np.float32)]
        for t in range(steps):
            host.append((0.9 * host[-1] + 0.45 * rng.standard_normal((n, d))).astype(np.float32))
        arrs = [_cuda(h) for h in host]
    else:
        host = [(rng.standard_t(4, size=(n, d)) * 0.1).astype(np.float32) for _ in range(steps + 1)]
        arrs = [_cuda(h) for h in host]
        Ds = [_cuda((np.sum(h.astype(np.float64) ** 2, axis=1) * rng.uniform(0.05, 2.0, n))) for h in host]
    torch.cuda.synchronize()
    outs = []
    for flags in (0, E.FLAG_OVERLAP):
        if mode == "grad":
            eng = E.AdaCGD(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=0.4, master_levels=ml,
                           grad_mode=E.GRAD_EXTERNAL, x0=x0, grad0=arrs[0], flags=flags | E.FLAG_RETAIN_EXT)
        else:
            eng = E.AdaCGD(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=1.0, master_levels=ml,
                           grad_mode=E.DIFF_EXTERNAL, init_mode=E.INIT_ZERO, x0=x0, flags=flags | any_order)
        levels = []
        for t in range(1, steps + 1):
            if mode == "grad":
                eng.step(arrs[t])
            else:
                eng.step(arrs[t], Ds[t])
            if t in (3, steps):
                levels.append(eng.state(E.F_LEVEL).tolist())
        outs.append((levels, eng.state(E.F_X), eng.state(E.F_G), eng.state(E.F_GTILDE), eng.state(E.F_GI),
                     eng.state(E.F_MSG_IDX), eng.state(E.F_MSG_VAL), eng.state(E.F_LEVEL_HIST)))
        eng.close()
    assert outs[0][0] == outs[1][0]
    if mode == "diff_quant":
        hist = outs[1][7]
        assert sum(int(hist[j]) for j in range(1, len(wl) + 1) if wl[j - 1][0] == O.QUANT) > 0, hist   # dense messages were aggregated
        assert sum(int(hist[j]) for j in range(1, len(wl) + 1) if wl[j - 1][0] == O.TOPK) > 0, hist
    if mode == "diff_block_rank":
        hist = outs[1][7]
        for kind in (O.RANK, O.QUANT_BLOCK):
            assert sum(int(hist[j]) for j in range(1, len(wl) + 1) if wl[j - 1][0] == kind) > 0, (kind, hist)
    for a, b in zip(outs[0][1:], outs[1][1:]):
        assert np.array_equal(np.ascontiguousarray(a).view(np.uint8), np.ascontiguousarray(b).view(np.uint8))
    if mode == "grad":
        orc = O.AdaCGDOracle(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=0.4, master_levels=ml)
        orc.init(np.zeros(d, dtype=np.float32), host[0], O.INIT_FULLGRAD)
        for t in range(1, steps + 1):
            orc.step(grads=host[t])
        assert np.array_equal(bits(outs[1][1]), bits(orc.x))
        assert np.array_equal(bits(outs[1][4]), bits(orc.gi))
        assert outs[1][7].tolist() == orc.level_hist_w.tolist()


def _run_external(n, d, wl, zw, ml, zm, steps, seed, tag):
    """Drives engine and oracle with the same supplied gradients and compares every step."""
    E = _eng()
    rng = np.random.default_rng(seed)
    grads = [rng.standard_normal((n, d)).astype(np.float32)]
    for t in range(steps):      # drifting gradients whose step-to-step change varies over two decades
        s = np.float32(10.0 ** rng.uniform(-2, 0))
        grads.append((grads[-1] + s * rng.standard_normal((n, d))).astype(np.float32))
    x0 = rng.standard_normal(d).astype(np.float32)
    orc = O.AdaCGDOracle(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=zw, master_levels=ml, zeta_master=zm)
    orc.init(x0, grads[0], O.INIT_FULLGRAD)
    eng = E.AdaCGD(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=zw, master_levels=ml, zeta_master=zm,
                   grad_mode=E.GRAD_EXTERNAL, x0=_cuda(x0), grad0=_cuda(grads[0]))
    mlev = []
    with until_near_tie(tag):
        for t in range(1, steps + 1):
            res, rm = orc.step(grads=grads[t])
            if rm is not None:
                mlev.append(rm.level)
            eng.step(_cuda(grads[t]))
            compare_step(eng, orc, res, rm, (tag, t))
        hist_w = eng.state(E.F_LEVEL_HIST)
        assert hist_w.tolist() == orc.level_hist_w.tolist()
    eng.close()
    for t in range(orc.t + 1, steps + 1):        # (a run cut short at a near tie: the oracle finishes alone)
        res, rm = orc.step(grads=grads[t])
        if rm is not None:
            mlev.append(rm.level)
    return orc, mlev


@pytest.mark.parametrize("zm", [0.3, 1.0, 4.0])
def test_adaptive_master_bit_exact(zm):
    """Server-side adaptive compressor (Corollary on bidirectional Ada3PC, Section 4.3): several
    master levels with a positive trigger constant, including steps where the master sends
    nothing.  Every master decision, message and the broadcast estimator g match the oracle."""
    n, d = 3, 3 * 8192 + 516
    wl = [(O.TOPK, 8), (O.TOPK, 300), (O.TOPK, 4000), (O.TOPK, d // 2)]
    ml = [(O.TOPK, 4), (O.TOPK, 120), (O.QUANT, 4), (O.TOPK, 2500), (O.TOPK, d)]
    orc, mlev = _run_external(n, d, wl, 1.5, ml, zm, 8, 77, ("ada-master", zm))
    assert len(set(mlev)) >= 2, mlev          # the master did adapt over the run
    assert orc.level_hist_m.sum() == 8


@pytest.mark.parametrize("name", ["gd", "ef21_top1", "clag", "lag"])
def test_special_cases_bit_exact(name):
    """The methods AdaCGD reduces to (Section 4.3: one level -> CLAG, zeta = 0 -> EF21,
    identity level -> LAG / plain GD) run through the same kernels and match the oracle."""
    n, d = 3, 2 * 8192 + 516
    wl, zw = {"gd": ([(O.TOPK, d)], 0.0), "ef21_top1": ([(O.TOPK, 1)], 0.0),
              "clag": ([(O.TOPK, 200)], 1.5), "lag": ([(O.TOPK, d)], 1.5)}[name]
    ml = [(O.TOPK, d)]                         # identity on the server: unidirectional compression
    orc, _ = _run_external(n, d, wl, zw, ml, 0.0, 6, 5, name)
    if name == "gd":                           # every worker sends everything at every step
        assert orc.level_hist_w.tolist() == [0, 6 * n]
    if name == "ef21_top1":
        assert orc.level_hist_w.tolist() == [0, 6 * n]
    if name in ("clag", "lag"):
        assert orc.level_hist_w[0] > 0          # some communications were skipped


def test_largest_dimension_properties():
    """d just above 2^30 (every per-worker array crosses 4 GiB), one worker, one step.  The oracle's
    full sort is out of reach at this size, so what is unique about the result is checked
    instead, with torch reductions on the device: the message is the exact Top-K support (sorted,
    K entries, values equal to v there, nothing outside exceeds the smallest value inside), the
    estimator is h + C(v) bit for bit, and S, D and the chosen level's error match fp64 sums."""
    E = _eng()
    import torch
    d = (1 << 30) + 3 * 8192 + 4
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20221100188)
    g0 = torch.randn(1, d, dtype=torch.float32, device="cuda", generator=gen)
    g1 = g0 + 0.3 * torch.randn(1, d, dtype=torch.float32, device="cuda", generator=gen)
    wl = [(O.TOPK, 16), (O.TOPK, d // 1000), (O.TOPK, d // 50)]
    zeta = 0.5
    x0 = torch.zeros(d, dtype=torch.float32, device="cuda")
    KM = d // 400
    eng = E.AdaCGD(n=1, d=d, gamma=0.05, worker_levels=wl, zeta_worker=zeta, master_levels=[(O.TOPK, KM)],
                   zeta_master=0.0, grad_mode=E.GRAD_EXTERNAL, init_mode=E.INIT_ZERO, x0=x0, grad0=g0,
                   flags=E.FLAG_RETAIN_EXT)
    eng.step(g1)
    lev = int(eng.state(E.F_LEVEL)[0])
    S, D, err = eng.state(E.F_SQNORM)[0], eng.state(E.F_D)[0], eng.state(E.F_ERR)[0]
    v = g1[0]                                    # h = 0: the compressor's argument is the gradient itself
    S_ref = float(torch.sum(v.double() ** 2))
    D_ref = float(torch.sum((g1[0].double() - g0[0].double()) ** 2))
    assert abs(S - S_ref) <= 1e-10 * S_ref and abs(D - D_ref) <= 1e-10 * D_ref
    assert lev >= 1 and S > zeta * D
    assert np.all(np.diff(err) <= 0)             # larger K, smaller error
    for j in range(1, lev):
        assert err[j - 1] > zeta * D             # the cascade went past these levels
    assert lev == len(wl) or err[lev - 1] <= zeta * D
    K = wl[lev - 1][1]
    idx, val = eng.messages()[0]
    assert len(idx) == K and np.all(np.diff(idx) > 0) and idx[0] >= 0 and idx[-1] < d
    tidx = torch.from_numpy(idx.astype(np.int64)).cuda()
    tval = torch.from_numpy(val).cuda()
    assert torch.equal(v[tidx].view(torch.int32), tval.view(torch.int32))
    rest = v.abs()
    rest[tidx] = 0
    assert float(rest.max()) <= float(tval.abs().min())
    sent = float(torch.sum(tval.double() ** 2))
    assert abs(err[lev - 1] - (S_ref - sent)) <= 1e-9 * S_ref
    expect = torch.zeros(d, dtype=torch.float32, device="cuda")
    expect[tidx] = tval
    del rest
    gi = torch.from_numpy(eng.state(E.F_GI)[0]).cuda()
    assert torch.equal(gi.view(torch.int32), expect.view(torch.int32))
    del gi
    # server: with one worker and zero initial estimators g~ = the message, and the master sends
    # the Top-KM entries of it (g = 0 before): a subset of the worker's message
    assert np.array_equal(bits(eng.state(E.F_GTILDE)), bits(expect.cpu().numpy()))
    midx, mval = eng.state(E.F_M_MSG_IDX), eng.state(E.F_M_MSG_VAL)
    assert int(eng.state(E.F_M_LEVEL)[0]) == 1 and len(midx) == KM and np.all(np.diff(midx) > 0)
    tm = torch.from_numpy(midx.astype(np.int64)).cuda()
    tmv = torch.from_numpy(mval).cuda()
    assert torch.equal(expect[tm].view(torch.int32), tmv.view(torch.int32))
    rest = expect.abs()
    rest[tm] = 0
    assert float(rest.max()) <= float(tmv.abs().min())
    g = torch.zeros(d, dtype=torch.float32, device="cuda")
    g[tm] = tmv
    assert np.array_equal(bits(eng.state(E.F_G)), bits(g.cpu().numpy()))
    eng.close()


def test_many_workers_small_dimension():
    """n in the thousands (one grid row per worker), d below one wavefront's share: every kernel's
    per-node bookkeeping at the other extreme of the shapes."""
    n, d = 3000, 130
    wl = [(O.TOPK, 1), (O.TOPK, 13), (O.TOPK, 65), (O.QUANT, 4), (O.TOPK, d)]
    ml = [(O.TOPK, 7), (O.TOPK, 40)]
    orc, _ = _run_external(n, d, wl, 1.2, ml, 0.7, 3, 11, "many-workers")
    assert (orc.level_hist_w > 0).sum() >= 3


@pytest.mark.parametrize("n,d,quant", [(4, 900, True), (3, 20000 + 13, True), (2, 140 * 8192 + 36, False),
                                       (3, 2 * 8192 + 517, False)])
def test_general_triggers_bit_exact(n, d, quant):
    """Conditions of the cascade from the wider family err_j <= zeta_j D + eta_j S (Section 4.2,
    Lemma 2 allow any), different at every position, on both sides; short vectors (one-block
    kernel), the two-pass sequence with a quantiser level, and the one-pass sequence."""
    E = _eng()
    rng = np.random.default_rng(31 * d + n)
    Ks = sorted({max(1, min(d, k)) for k in (2, d // 100, d // 16, d // 3)})
    wl = [(O.TOPK, k) for k in Ks]
    if quant:
        wl.insert(2, (O.QUANT, 4))
    wl.append((O.TOPK, d))
    ml = [(O.TOPK, max(1, d // 50)), (O.TOPK, max(2, d // 5))]
    steps = 5
    grads = [make_vectors(rng, n, d, "heavy") for _ in range(steps + 1)]
    for t in range(1, steps + 1):
        grads[t] = (grads[t - 1] + grads[t] * np.float32(10.0 ** rng.uniform(-1.5, 0))).astype(np.float32)
    x0 = rng.standard_normal(d).astype(np.float32)
    seen = set()
    for trial in range(3):
        tw = [(float(rng.uniform(0, 1.5)) * (trial > 0), float(rng.uniform(0.0, 0.5))) for _ in wl]
        tw[0] = (tw[0][0], float(rng.uniform(0, 0.2)))
        tm = [(float(rng.uniform(0, 2)), float(rng.uniform(0, 0.3))) for _ in ml]
        kw = dict(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=99.0, master_levels=ml, zeta_master=99.0,
                  worker_triggers=tw, master_triggers=tm, seed=5)
        orc = O.AdaCGDOracle(**kw)
        orc.init(x0, grads[0], O.INIT_ZERO)
        eng = E.AdaCGD(grad_mode=E.GRAD_EXTERNAL, init_mode=E.INIT_ZERO, x0=_cuda(x0), grad0=_cuda(grads[0]),
                       flags=E.FLAG_ANY_LEVEL_ORDER, **kw)
        with until_near_tie((n, d, trial)):
            for t in range(1, steps + 1):
                res, rm = orc.step(grads=grads[t])
                eng.step(_cuda(grads[t]))
                compare_step(eng, orc, res, rm, (n, d, trial, t))
                seen.update(r.level for r in res)
            assert eng.state(E.F_LEVEL_HIST).tolist() == orc.level_hist_w.tolist()
            assert eng.state(E.F_M_LEVEL_HIST).tolist() == orc.level_hist_m.tolist()
        eng.close()
    assert len(seen) >= 3, seen


def _csr_engine(wl, csr, x0=None, **kw):
    E = _eng()
    x0 = _cuda(np.zeros(wl.d, dtype=np.float32) if x0 is None else x0)
    return E.AdaCGD(n=wl.n, d=wl.d, gamma=wl.gamma, lam=wl.lam, worker_levels=wl.worker_levels,
                    zeta_worker=wl.zeta_worker, master_levels=wl.master_levels, zeta_master=wl.zeta_master,
                    grad_mode=E.GRAD_LOGISTIC_CSR, labels=_cuda(wl.labels), shard_offsets=wl.shard_offsets,
                    csr=csr, x0=x0, **kw)


def _sparsify(wl, density, rng, binary):
    """Keeps a random subset of the entries of a dense workload (some rows and columns end up
    empty); `binary` replaces the kept entries by 1."""
    keep = rng.random(wl.A.shape) < density
    keep[rng.integers(0, wl.A.shape[0], 3)] = False          # empty rows
    keep[:, rng.integers(0, wl.d, 2)] = False                # empty columns
    wl.A = np.where(keep, np.float32(1) if binary else wl.A, np.float32(0)).astype(np.float32)
    if wl.A.shape[1] > 3:
        wl.A[:, 3] = 1 if binary else wl.A[:, 3] + 2         # a dense column: long per-column lists
    return wl


@pytest.mark.parametrize("n,d,N,density,binary", [(4, 100, 64, 0.1, False), (3, 101, 50, 0.5, True),
                                                  (5, 8192 + 12, 7, 0.02, False), (2, 300, 2500, 0.04, True),
                                                  (2, 1500, 40, 0.6, False), (2, 40, 1200, 0.5, False)])
def test_sparse_gradient_kernel_matches_oracle(n, d, N, density, binary):
    """grad f_i(x) from compressed sparse rows against the oracle on the same matrix stored
    densely: both accumulate in fp64 and round once, so values agree to one fp32 unit in the
    last place (the sparse kernels add the stored entries only, in another order)."""
    E = _eng()
    rng = np.random.default_rng(7 * d + N)
    wl = _sparsify(W.tiny(seed=22, n=n, d=d, N=N), density, rng, binary)
    csr = W.to_csr(wl.A, binary)
    for scale in (0.0, 0.05, 3.0):
        x0 = (scale * rng.standard_normal(d)).astype(np.float32)
        eng = _csr_engine(wl, csr, x0=x0)
        got = eng.state(E.F_GRAD)
        eng.close()
        ref = np.stack([O.logistic_grad(A, y, x0, np.float64(np.float32(wl.lam)), np.float32) for A, y in wl.shards()])
        # sums of equal terms of both signs cancel to a residue at the fp64 rounding level (1e-18 next
        # to terms of 1e-2) whose value depends on the order: one fp32 unit, or that residue
        ulp = np.maximum(np.spacing(np.abs(ref)).astype(np.float64), 1e-15)
        assert np.all(np.abs(got.astype(np.float64) - ref.astype(np.float64)) <= ulp)
        assert_close_rel(got, ref, TRAJ_RTOL, ("grad", n, d, N, scale))
        if scale > 0:
            assert np.mean(bits(got) != bits(ref)) < 0.01


def test_trajectory_sparse_logreg_from_sparse_rows():
    """The binary-feature workload run from its compressed sparse rows: same bars as the dense run."""
    E = _eng()
    wl = W.sparse_logreg(T=300)
    orc = _logistic_oracle(wl)
    eng = _csr_engine(wl, W.to_csr(wl.A, binary=True))
    assert_close_rel(eng.state(E.F_GRAD), orc.y, TRAJ_RTOL, "grad0")
    for t in range(wl.T):
        orc.step()
        eng.step()
        if (t + 1) % 10 == 0:
            assert_close_rel(eng.state(E.F_X), orc.x, TRAJ_RTOL, ("x", t))
            assert_close_rel(eng.state(E.F_GRAD), orc.y, TRAJ_RTOL, ("grad", t))
            assert_close_rel(eng.state(E.F_G), orc.g, TRAJ_RTOL, ("g", t))
    assert eng.state(E.F_LEVEL_HIST).tolist() == orc.level_hist_w.tolist()
    eng.close()


def test_trajectory_sparse_features_reduced():
    """The sparse-rows workload of the benchmark at a size the oracle handles (dense copy made here)."""
    E = _eng()
    wl = W.sparse_features(n=6, d=8192 + 128, N=40, per_row=16, T=25)
    row_ptr, col, _ = wl.csr
    A = np.zeros((wl.labels.shape[0], wl.d), dtype=np.float32)
    A[np.repeat(np.arange(A.shape[0]), np.diff(row_ptr)), col] = 1
    wl.A = A
    orc = _logistic_oracle(wl)
    eng = _csr_engine(wl, wl.csr)
    assert_close_rel(eng.state(E.F_GRAD), orc.y, TRAJ_RTOL, "grad0")
    for t in range(wl.T):
        orc.step()
        eng.step()
        assert_close_rel(eng.state(E.F_X), orc.x, TRAJ_RTOL, ("x", t))
        assert_close_rel(eng.state(E.F_GRAD), orc.y, TRAJ_RTOL, ("grad", t))
        assert_close_rel(eng.state(E.F_G), orc.g, TRAJ_RTOL, ("g", t))
    assert eng.state(E.F_LEVEL_HIST).tolist() == orc.level_hist_w.tolist()
    assert (orc.level_hist_w > 0).sum() >= 2
    eng.close()


@pytest.mark.parametrize("n,d", [(4, 700), (3, 2 * 8192 + 516), (2, 130 * 8192)])
def test_compressed_initial_estimators_bit_exact(n, d):
    """g~_i^0 = Top-K(grad f_i(x^0)) with the last level's K (the CLAG / EF21 start), then a few steps."""
    E = _eng()
    rng = np.random.default_rng(d + n)
    wl = [(O.TOPK, max(1, d // 200)), (O.TOPK, max(2, d // 20))]
    grads = [make_vectors(rng, n, d, "heavy") for _ in range(4)]
    grads[0][0, : d // 2] = 0.0                        # a gradient with many zeros
    grads[0][1] = 0.0                                  # fewer non-zeros than K: zeros of both signs are selected,
    grads[0][1, ::3] = -0.0                            # and g~_i^0 = C(grad) keeps the sign of each
    grads[0][1, min(5, d - 1)] = 1.0
    if n > 2:
        grads[0][2] = 0.0                              # ... and one that is zero, with zeros of both signs: the
        grads[0][2, 1::2] = -0.0                       # level applies all the same and keeps K of them as they are
    for t in range(1, 4):
        grads[t] = (grads[t - 1] + grads[t] * np.float32(0.2)).astype(np.float32)
    x0 = rng.standard_normal(d).astype(np.float32)
    orc = O.AdaCGDOracle(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=1.0)
    orc.init(x0, grads[0], O.INIT_COMPRESSED)
    eng = E.AdaCGD(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=1.0, grad_mode=E.GRAD_EXTERNAL,
                   init_mode=E.INIT_COMPRESSED, x0=_cuda(x0), grad0=_cuda(grads[0]))
    assert np.array_equal(bits(eng.state(E.F_GI)), bits(orc.gi))
    assert np.array_equal(bits(eng.state(E.F_GTILDE)), bits(orc.gt))
    assert np.array_equal(bits(eng.state(E.F_G)), bits(orc.g))
    assert eng.state(E.F_LEVEL_HIST).sum() == 0 and eng.state(E.F_MSG_COUNT).sum() == 0
    with until_near_tie(("compressed start", n, d)):
        for t in range(1, 4):
            res, rm = orc.step(grads=grads[t])
            eng.step(_cuda(grads[t]))
            compare_step(eng, orc, res, rm, (n, d, t))
        assert eng.state(E.F_LEVEL_HIST).tolist() == orc.level_hist_w.tolist()
    eng.close()


def test_sparse_rows_degenerate_shapes():
    """No stored entry at all (the gradient is the regulariser's), and one row per worker with d = 1."""
    E = _eng()
    wl = W.tiny(seed=3, n=3, d=37, N=5)
    wl.A[:] = 0
    x0 = np.linspace(-2, 2, wl.d).astype(np.float32)
    eng = _csr_engine(wl, (np.zeros(wl.A.shape[0] + 1, dtype=np.int64), np.zeros(0, dtype=np.int32), None), x0=x0)
    ref = np.stack([O.logistic_grad(A, y, x0, np.float64(np.float32(wl.lam)), np.float32) for A, y in wl.shards()])
    assert np.array_equal(bits(eng.state(E.F_GRAD)), bits(ref))
    eng.step(nsteps=3)
    eng.close()
    wl = W.tiny(seed=4, n=2, d=1, N=1)
    wl.worker_levels, wl.master_levels = [(O.TOPK, 1)], []
    x0 = np.array([0.7], dtype=np.float32)
    eng = _csr_engine(wl, W.to_csr(wl.A), x0=x0)
    ref = np.stack([O.logistic_grad(A, y, x0, np.float64(np.float32(wl.lam)), np.float32) for A, y in wl.shards()])
    assert_close_rel(eng.state(E.F_GRAD), ref, TRAJ_RTOL, "d = 1")
    orc = _logistic_oracle(wl, x0=x0)
    for t in range(5):
        orc.step()
        eng.step()
        assert_close_rel(eng.state(E.F_X), orc.x, TRAJ_RTOL, ("x", t))
    eng.close()


@pytest.mark.parametrize("master", [True, False])
@pytest.mark.parametrize("n", [5, 70])
def test_overlap_mode_short_vectors(n, master):
    """Overlap mode on the one-block path (with and without the aggregation done by the workers' launch,
    with and without a master compressor): same results as the oracle, step by step."""
    E = _eng()
    d = 700
    rng = np.random.default_rng(n)
    wl = [(O.TOPK, 3), (O.TOPK, 40), (O.TOPK, 300)]
    ml = [(O.TOPK, 50)] if master else []
    grads = [rng.standard_normal((n, d)).astype(np.float32)]
    for t in range(8):
        grads.append((grads[-1] + np.float32(10.0 ** rng.uniform(-2, 0)) * rng.standard_normal((n, d))).astype(np.float32))
    x0 = rng.standard_normal(d).astype(np.float32)
    orc = O.AdaCGDOracle(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=1.0, master_levels=ml, zeta_master=0.5)
    orc.init(x0, grads[0], O.INIT_FULLGRAD)
    arrs = [_cuda(g) for g in grads]
    eng = E.AdaCGD(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=1.0, master_levels=ml, zeta_master=0.5,
                   grad_mode=E.GRAD_EXTERNAL, x0=_cuda(x0), grad0=arrs[0], flags=E.FLAG_OVERLAP | E.FLAG_RETAIN_EXT)
    with until_near_tie(("overlap, short", n, master)):
        for t in range(1, 9):
            res, rm = orc.step(grads=grads[t])
            eng.step(arrs[t])
            if min_margin(res + ([rm] if rm is not None else [])) < 1e-12:
                raise NearTie(repr((n, master, t)))      # also at the steps that are not compared
            if t % 3 == 0 or t == 8:
                compare_step(eng, orc, res, rm, (n, master, t))
        assert eng.state(E.F_LEVEL_HIST).tolist() == orc.level_hist_w.tolist()
    eng.close()


@pytest.mark.parametrize("n,d,flags", [(4, 900, 0), (3, 3 * 8192 + 516, 0), (2, 130 * 8192, 0), (3, 20000, "retain"),
                                       (3, 64 * 320, "block_rank")])
def test_checkpoint_and_restore_continue_bit_for_bit(n, d, flags):
    """State copied out after three steps and restored into a context that was initialised from other
    data continues exactly like the uninterrupted run (mixed level set: the Philox counter is part of it)."""
    E = _eng()
    rng = np.random.default_rng(d)
    wl = by_alpha([(O.TOPK, max(1, d // 300)), (O.QUANT, 4), (O.TOPK, max(2, d // 10))], d)
    if d >= 130 * 8192:
        wl = [(O.TOPK, d // 300), (O.TOPK, d // 10)]              # one-pass sequence
    if flags == "block_rank":       # block-wise quantiser and Rank-K levels: nothing of theirs outlives a step
        wl = [(O.RANK, (2, 64)), (O.TOPK, d // 300), (O.QUANT_BLOCK, (4, 256)), (O.RANK, (40, 64)), (O.TOPK, d // 10)]
    ml = [(O.TOPK, max(1, d // 50))]
    grads = [make_vectors(rng, n, d, "normal") for _ in range(7)]
    for t in range(1, 7):
        grads[t] = (grads[t - 1] + grads[t] * np.float32(0.3)).astype(np.float32)
    arrs = [_cuda(g) for g in grads]
    x0 = rng.standard_normal(d).astype(np.float32)
    fl = E.FLAG_RETAIN_EXT if flags == "retain" else E.FLAG_ANY_LEVEL_ORDER if flags == "block_rank" else 0
    kw = dict(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=1.0, master_levels=ml, zeta_master=0.3,
              grad_mode=E.GRAD_EXTERNAL, seed=9, flags=fl)
    a = E.AdaCGD(x0=_cuda(x0), grad0=arrs[0], **kw)
    for t in range(1, 4):
        a.step(arrs[t])
    ck = a.checkpoint()
    for t in range(4, 7):
        a.step(arrs[t])
    b = E.AdaCGD(x0=_cuda(np.zeros(d, dtype=np.float32)), grad0=arrs[5], **kw)
    b.step(arrs[6])                                                # some unrelated history
    b.restore(ck)
    assert int(b.state(E.F_STEP)[0]) == 3
    for t in range(4, 7):
        b.step(arrs[t])
    for f in E.AdaCGD.CHECKPOINT_FIELDS + (E.F_LEVEL, E.F_MSG_IDX, E.F_MSG_VAL, E.F_ERR, E.F_COMM):
        fa, fb = a.state(f), b.state(f)
        assert np.array_equal(np.ascontiguousarray(fa).view(np.uint8), np.ascontiguousarray(fb).view(np.uint8)), f
    with pytest.raises(E.AdaCGDError) as ei:
        b.set_state(E.F_LEVEL, np.zeros(n, dtype=np.int32))
    assert ei.value.code == 6
    with pytest.raises(E.AdaCGDError) as ei:
        b.set_state(E.F_X, np.zeros(d + 1, dtype=np.float32))
    assert ei.value.code == 6
    a.close()
    b.close()


def test_stored_trajectory_from_the_engine():
    """The stored trajectory (tests/golden, written from the oracle) out of the HIP path."""
    import importlib.util
    import os
    E = _eng()
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_trajectory_golden", os.path.join(here, "make_trajectory_golden.py"))
    G = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(G)
    stored = open(os.path.join(here, "trajectory_tiny_external.txt")).read().splitlines()
    x0, grads = G.inputs()
    eng = E.AdaCGD(n=G.N, d=G.D, gamma=G.GAMMA, worker_levels=G.WORKER_LEVELS, zeta_worker=G.ZETA_W,
                   master_levels=G.MASTER_LEVELS, zeta_master=G.ZETA_M, seed=G.SEED, grad_mode=E.GRAD_EXTERNAL,
                   x0=_cuda(x0), grad0=_cuda(grads[0]), flags=E.FLAG_ANY_LEVEL_ORDER)   # the 4-bit level sits before Top-25
    for t in range(1, G.STEPS + 1):
        eng.step(_cuda(grads[t]))
        msgs = ";".join(",".join(str(int(i)) for i in m[0]) for m in eng.messages())
        line = "%d | %s | %d | %s | %s %s %s %s" % (
            t, " ".join(str(int(v)) for v in eng.state(E.F_LEVEL)), int(eng.state(E.F_M_LEVEL)[0]), msgs,
            G.digest(eng.state(E.F_X)), G.digest(eng.state(E.F_G)), G.digest(eng.state(E.F_GTILDE)),
            G.digest(eng.state(E.F_GI)))
        assert line == stored[t], t
    eng.close()


@pytest.mark.parametrize("bits_", [(4,), (2, 8), (2, 4, 8), (2, 3, 4, 6, 8)])
def test_one_to_five_quantiser_levels_bit_exact(bits_):
    """Level sets with one, two, three (kernels specialised on the count) and five (general kernel)
    quantiser levels next to two Top-K sizes, on the 16-byte vector path."""
    E = _eng()
    n, d = 4, 3 * 8192 + 516
    rng = np.random.default_rng(len(bits_))
    wl = by_alpha([(O.TOPK, 50), (O.TOPK, 3000)] + [(O.QUANT, b) for b in bits_], d)
    grads = [make_vectors(rng, n, d, "heavy") for _ in range(5)]
    for t in range(1, 5):
        grads[t] = (grads[t - 1] + grads[t] * np.float32(10.0 ** rng.uniform(-2, 0))).astype(np.float32)
    x0 = rng.standard_normal(d).astype(np.float32)
    kw = dict(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=0.05, master_levels=[(O.TOPK, 500)], zeta_master=0.0,
              seed=77)
    orc = O.AdaCGDOracle(**kw)
    orc.init(x0, grads[0], O.INIT_ZERO)
    eng = E.AdaCGD(grad_mode=E.GRAD_EXTERNAL, init_mode=E.INIT_ZERO, x0=_cuda(x0), grad0=_cuda(grads[0]), **kw)
    with until_near_tie(("quantiser levels", bits_)):
        for t in range(1, 5):
            res, rm = orc.step(grads=grads[t])
            eng.step(_cuda(grads[t]))
            compare_step(eng, orc, res, rm, (bits_, t))       # includes the realised error of every quantiser level
    eng.close()


def test_two_contexts_interleaved_on_two_streams():
    """Two engines with different shapes, each on a stream of its own, stepped alternately without
    synchronisation in between: each matches its own oracle (the library keeps no state outside a context)."""
    E = _eng()
    import torch
    specs = [(5, 900, [(O.TOPK, 9), (O.TOPK, 300)], 11), (3, 2 * 8192 + 516, [(O.TOPK, 40), (O.QUANT, 4), (O.TOPK, 5000)], 12)]
    runs = []
    for n, d, wl, seed in specs:
        rng = np.random.default_rng(seed)
        wl = by_alpha(wl, d)
        grads = [make_vectors(rng, n, d, "normal") for _ in range(6)]
        for t in range(1, 6):
            grads[t] = (grads[t - 1] + grads[t] * np.float32(0.3)).astype(np.float32)
        x0 = rng.standard_normal(d).astype(np.float32)
        kw = dict(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=1.0, master_levels=[(O.TOPK, max(1, d // 40))],
                  zeta_master=0.2, seed=seed)
        orc = O.AdaCGDOracle(**kw)
        orc.init(x0, grads[0], O.INIT_FULLGRAD)
        st = torch.cuda.Stream()
        arrs = [_cuda(g) for g in grads]
        torch.cuda.synchronize()
        eng = E.AdaCGD(grad_mode=E.GRAD_EXTERNAL, x0=_cuda(x0), grad0=arrs[0], stream=st.cuda_stream, **kw)
        runs.append((eng, orc, grads, arrs))
    for t in range(1, 6):
        for eng, orc, grads, arrs in runs:
            eng.step(arrs[t])
    for eng, orc, grads, arrs in runs:
        with until_near_tie(("interleaved", orc.d)):
            for t in range(1, 6):
                res, rm = orc.step(grads=grads[t])
                if min_margin(res + [rm]) < 1e-12:
                    raise NearTie(repr(("interleaved", orc.d, t)))
            compare_step(eng, orc, res, rm, ("interleaved", orc.d))
            assert eng.state(E.F_LEVEL_HIST).tolist() == orc.level_hist_w.tolist()
        eng.close()


@pytest.mark.parametrize("dense", [False, True])
def test_aggregation_with_wide_exponent_spread(dense):
    """Messages that put values more than 2^30 apart in magnitude on the same coordinate (per-worker scales
    from 1e-12 to 1e+12).  The oracle adds the messages of a coordinate in ascending worker index in fp64;
    for Top-K level sets with up to 64 workers so does the aggregation kernel, and the results agree bit for
    bit whatever the data (a hundred coordinates here carry values whose sum in another order would differ
    already in fp32).  Dense quantised messages are added as partial sums in a fixed other order, which can
    differ in the last place of the fp64 sum once the exponents spread over more than 53 - 24 bits; the
    aggregate is that sum divided by n, added to the old value and rounded to fp32, 29 bits coarser, and
    must still agree bit for bit on data like these."""
    E = _eng()
    n, d = 12, 3 * 8192 + 516
    rng = np.random.default_rng(2030)
    scales = (10.0 ** rng.permutation(np.linspace(-12, 12, n))).astype(np.float32)
    wl = [(O.QUANT, 8)] if dense else [(O.TOPK, d)]
    steps = 4
    x0 = np.zeros(d, dtype=np.float32)
    if dense:
        orc = O.AdaCGDOracle(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=0.0, master_levels=[], seed=17)
        orc.init(x0, None, O.INIT_ZERO)
        eng = E.AdaCGD(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=0.0, master_levels=[],
                       grad_mode=E.DIFF_EXTERNAL, init_mode=E.INIT_ZERO, x0=_cuda(x0), seed=17)
    else:
        g0 = np.zeros((n, d), dtype=np.float32)
        orc = O.AdaCGDOracle(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=0.0, master_levels=[])
        orc.init(x0, g0, O.INIT_ZERO)
        eng = E.AdaCGD(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=0.0, master_levels=[],
                       grad_mode=E.GRAD_EXTERNAL, init_mode=E.INIT_ZERO, x0=_cuda(x0), grad0=_cuda(g0))
    with until_near_tie(("wide spread", dense)):
        for t in range(1, steps + 1):
            v = (rng.standard_normal((n, d)) * scales[:, None]).astype(np.float32)
            if not dense:
                # coordinates whose fp64 sum depends on the order of the additions, visibly in fp32:
                # ((1 + 2^-60) - 1) + 2^-60 = 2^-60 in ascending worker order, 2^-59 if the two ones meet first
                v[:, :100] = 0.0
                v[0, :100], v[1, :100], v[2, :100], v[3, :100] = 1.0, 2.0 ** -60, -1.0, 2.0 ** -60
            if dense:
                D = np.ones(n)
                res, rm = orc.step(diffs=v, D=D)
                eng.step(_cuda(v), _cuda(D))
            else:
                res, rm = orc.step(grads=v)
                eng.step(_cuda(v))
            assert all(r.level == 1 for r in res)
            compare_step(eng, orc, res, rm, ("wide spread", dense, t), check_master=False)
    lo, hi = np.abs(orc.gt[orc.gt != 0]).min(), np.abs(orc.gt).max()
    assert hi > 1e9                                   # the large workers dominate the aggregate
    eng.close()


@pytest.mark.parametrize("n,d,flags", [(4, 3 * 8192 + 516, 0), (3, 2 * 8192 + 517, 0), (5, 1000, 0), (2, 4095, 0),
                                       (3, 1000, "two_pass"), (2, 130, 0), (2, 5 * 8192, 0)])
@pytest.mark.parametrize("blocks", [((4, 256),), ((8, 64), (2, 2048)), ((4, 128), (4, 1024), (3, 512))])
def test_block_wise_quantiser_levels_bit_exact(n, d, flags, blocks):
    """Level sets with block-wise b-bit quantisers (one max-norm scale per block of B coordinates) next to
    Top-K levels and a plain quantiser, on the 16-byte and the scalar path, the one-block kernel and the
    general kernels, worker and master side: levels, errors, estimators, codes and per-block scales."""
    E = _eng()
    rng = np.random.default_rng(d + 7 * len(blocks))
    wl = [(O.TOPK, max(1, d // 300)), (O.TOPK, max(2, d // 20))] + [(O.QUANT_BLOCK, bb) for bb in blocks]
    if len(blocks) == 2:
        wl.append((O.QUANT, 4))
    wl = by_alpha(wl, d)
    ml = by_alpha([(O.TOPK, max(1, d // 100)), (O.QUANT_BLOCK, (4, 64))], d)
    steps = 4
    grads = [make_vectors(rng, n, d, "heavy") for _ in range(steps + 1)]
    for g in grads:                                   # blocks of very different size, one block of zeros
        g[:, : min(d, 64)] *= np.float32(1e-6)
        g[:, min(d, 64): min(d, 128)] = 0.0
    for t in range(1, steps + 1):
        grads[t] = (grads[t - 1] + grads[t] * np.float32(10.0 ** rng.uniform(-2, 0))).astype(np.float32)
    x0 = rng.standard_normal(d).astype(np.float32)
    seen = set()
    for zeta in (0.0, 0.05, 0.8):
        kw = dict(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=zeta, master_levels=ml, zeta_master=0.3, seed=41)
        orc = O.AdaCGDOracle(**kw)
        orc.init(x0, grads[0], O.INIT_ZERO)
        eng = E.AdaCGD(grad_mode=E.GRAD_EXTERNAL, init_mode=E.INIT_ZERO, x0=_cuda(x0), grad0=_cuda(grads[0]),
                       flags=(E.FLAG_TWO_PASS if flags == "two_pass" else 0) | E.FLAG_ANY_LEVEL_ORDER, **kw)
        with until_near_tie(("block-wise", n, d, blocks, zeta)):
            for t in range(1, steps + 1):
                res, rm = orc.step(grads=grads[t])
                eng.step(_cuda(grads[t]))
                compare_step(eng, orc, res, rm, ("block-wise", n, d, blocks, zeta, t))
                codes = scales = None
                for i, r in enumerate(res):
                    if r.level > 0:
                        seen.add(wl[r.level - 1])
                    if r.scales is not None:
                        if codes is None:
                            codes, scales = eng.state(E.F_QCODES), eng.state(E.F_QBSCALE)
                        assert np.array_equal(codes[i].astype(np.int32), r.codes), (t, i)
                        assert np.array_equal(bits(scales[i][: len(r.scales)]), bits(r.scales)), (t, i)
            assert eng.state(E.F_LEVEL_HIST).tolist() == orc.level_hist_w.tolist()
            assert eng.state(E.F_M_LEVEL_HIST).tolist() == orc.level_hist_m.tolist()
            assert eng.state(E.F_COMM).tolist()[1] == sum(
                int(orc.level_hist_w[j]) * O.AdaCGDOracle.message_bits(j, wl, d) for j in range(len(wl) + 1))
        eng.close()
    assert any(k == O.QUANT_BLOCK for k, _ in seen), seen


def compare_step_rank(eng, orc, res, rm, tag, vmax):
    """Comparison of one step when the level set holds Rank-K levels.  The projector comes from an
    eigen-decomposition on one side and a library SVD on the other: the fp64 products X P agree to about
    1e-13 and are then rounded to fp32, so C(v) -- and with it the estimators and everything downstream --
    agrees bit for bit except where that difference straddles an fp32 rounding boundary (one unit in the
    last place, rarely; `vmax` = largest |v| per worker bounds what one such coordinate does to an error).
    Levels must agree; reductions to 1e-12, the Rank-K errors and spectrum to 1e-9;
    vectors to 1e-6 of their largest element with at most one coordinate in a thousand differing at all."""
    E = _eng()
    if min_margin(res + ([rm] if rm is not None else [])) < 1e-7:
        raise NearTie(repr(tag))
    lev = eng.state(E.F_LEVEL)
    S, D, err = eng.state(E.F_SQNORM), eng.state(E.F_D), eng.state(E.F_ERR)
    spec = eng.state(E.F_RANK_SPECTRUM)
    assert lev.tolist() == [r.level for r in res], (tag, "levels")
    for i, r in enumerate(res):
        assert abs(S[i] - r.S) <= RED_RTOL * max(r.S, 1e-300) and abs(D[i] - r.D) <= RED_RTOL * max(r.D, 1e-300), (tag, i)
        if r.level == 0:
            continue
        for j, e in enumerate(r.err):
            tol = (1e-9 if orc.wl[j][0] == O.RANK else RED_RTOL) * max(e, r.S * 1e-6, 1e-300)
            if orc.wl[j][0] == O.RANK:      # plus two coordinates whose fp32 rounding of C(v) falls the other way
                tol += 2 * 2.0 * np.sqrt(e) * 2.0 ** -23 * vmax[i]
            assert abs(err[i, j] - e) <= tol, (tag, i, j, err[i, j], e)
        if r.sigma is not None:
            lam = r.sigma.astype(np.float64) ** 2
            assert np.all(np.diff(spec[i]) <= 0)
            assert np.abs(spec[i] - lam).max() <= 1e-9 * lam[0], (tag, i, "spectrum")
    for name, got, want in (("g_i", eng.state(E.F_GI), orc.gi), ("g~", eng.state(E.F_GTILDE), orc.gt),
                            ("g", eng.state(E.F_G), orc.g), ("x", eng.state(E.F_X), orc.x)):
        assert_close_rel(got, want, 1e-6, (tag, name))
        assert np.mean(bits(got) != bits(want)) <= 1e-3, (tag, name, "coordinates that differ")
    if rm is not None:
        assert int(eng.state(E.F_M_LEVEL)[0]) == rm.level, (tag, "master level")


@pytest.mark.parametrize("n,rows,c,mode", [(3, 160, 16, "grad"), (2, 300, 32, "grad"), (2, 1000, 64, "grad"),
                                           (3, 4 * 8192 // 16 + 5, 16, "diff"), (1, 64, 64, "grad")])
def test_rank_k_levels_match_the_oracle(n, rows, c, mode):
    """Level sets with Rank-K levels (the argument read as a rows x c matrix, truncated SVD) next to Top-K
    levels, worker and master side, for every supported column count; gradients with a few dominant
    directions plus noise, so that the cascade stops at different ranks."""
    E = _eng()
    d = rows * c
    rng = np.random.default_rng(rows + c)
    wl = [(O.RANK, (1, c)), (O.TOPK, max(1, d // 40)), (O.RANK, (3, c)), (O.RANK, (c // 2, c)), (O.TOPK, d)]
    ml = [(O.RANK, (2, c)), (O.TOPK, max(1, d // 10))]

    def structured():
        k = 4
        X = (rng.standard_normal((n, rows, k)) * np.array([8.0, 4.0, 2.0, 1.0])) @ rng.standard_normal((n, k, c))
        return (X + 0.3 * rng.standard_normal((n, rows, c))).reshape(n, d).astype(np.float32)

    steps = 4
    grads = [structured() for _ in range(steps + 1)]
    for t in range(1, steps + 1):
        grads[t] = (grads[t - 1] + grads[t] * np.float32(10.0 ** rng.uniform(-1.5, 0))).astype(np.float32)
    x0 = rng.standard_normal(d).astype(np.float32)
    seen = set()
    for zeta in (0.0, 0.02, 0.3, 2.0):
        kw = dict(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=zeta, master_levels=ml, zeta_master=0.05)
        orc = O.AdaCGDOracle(**kw)
        if mode == "diff":
            orc.init(x0, None, O.INIT_ZERO)
            eng = E.AdaCGD(grad_mode=E.DIFF_EXTERNAL, init_mode=E.INIT_ZERO, x0=_cuda(x0), flags=E.FLAG_ANY_LEVEL_ORDER, **kw)
        else:
            orc.init(x0, grads[0], O.INIT_ZERO)
            eng = E.AdaCGD(grad_mode=E.GRAD_EXTERNAL, init_mode=E.INIT_ZERO, x0=_cuda(x0), grad0=_cuda(grads[0]),
                           flags=E.FLAG_ANY_LEVEL_ORDER, **kw)
        with until_near_tie(("rank", n, rows, c, mode, zeta)):
            for t in range(1, steps + 1):
                if mode == "diff":
                    Dt = np.sum(grads[t].astype(np.float64) ** 2, axis=1) * 10.0 ** rng.uniform(-2, 1, n)
                    res, rm = orc.step(diffs=grads[t], D=Dt)
                    eng.step(_cuda(grads[t]), _cuda(Dt))
                else:
                    res, rm = orc.step(grads=grads[t])
                    eng.step(_cuda(grads[t]))
                vmax = np.abs(grads[t]).max(axis=1) + np.abs(orc.gi).max(axis=1)
                compare_step_rank(eng, orc, res, rm, ("rank", n, rows, c, mode, zeta, t), vmax)
                seen.update(wl[r.level - 1] for r in res if r.level > 0)
                # put the engine's state into the oracle: later steps then start from identical vectors
                orc.gi, orc.gt, orc.gt_prev = eng.state(E.F_GI), eng.state(E.F_GTILDE), eng.state(E.F_GTILDE_PREV)
                orc.g, orc.x = eng.state(E.F_G), eng.state(E.F_X)
            assert eng.state(E.F_LEVEL_HIST).tolist() == orc.level_hist_w.tolist()
            assert eng.state(E.F_COMM).tolist()[1] == sum(
                int(orc.level_hist_w[j]) * O.AdaCGDOracle.message_bits(j, wl, d) for j in range(len(wl) + 1))
        eng.close()
    assert any(k == O.RANK for k, _ in seen), seen


def test_rank_k_levels_of_large_rank():
    """Ranks above half the column count (the projection kernels then hold all 64 eigenvectors in LDS, more
    than 64 KB of it), up to the full rank, whose message is the argument itself up to rounding."""
    E = _eng()
    n, rows, c = 2, 300, 64
    d = rows * c
    rng = np.random.default_rng(99)
    wl = [(O.RANK, (40, c)), (O.RANK, (57, c)), (O.RANK, (64, c))]
    X = (rng.standard_normal((n, rows, 6)) * np.array([9.0, 5.0, 3.0, 2.0, 1.5, 1.0])) @ rng.standard_normal((n, 6, c))
    v = (X + rng.standard_normal((n, rows, c)) * np.linspace(0.05, 1.0, c)).reshape(n, d).astype(np.float32)
    x0 = np.zeros(d, dtype=np.float32)
    for scale in (1e-4, 3e-3, 1e-12):          # the level the cascade stops at moves with the right-hand side
        kw = dict(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=1.0, master_levels=[], zeta_master=0.0)
        orc = O.AdaCGDOracle(**kw)
        orc.init(x0, None, O.INIT_ZERO)
        eng = E.AdaCGD(grad_mode=E.DIFF_EXTERNAL, init_mode=E.INIT_ZERO, x0=_cuda(x0), **kw)
        Dt = np.sum(v.astype(np.float64) ** 2, axis=1) * scale
        res, rm = orc.step(diffs=v, D=Dt)
        eng.step(_cuda(v), _cuda(Dt))
        with until_near_tie(("rank, large", scale)):
            compare_step_rank(eng, orc, res, None, ("rank, large", scale), np.abs(v).max(axis=1))
        if scale == 1e-12:
            assert eng.state(E.F_LEVEL).tolist() == [3] * n
            assert np.mean(bits(eng.state(E.F_GI)) != bits(v)) <= 1e-3          # full rank: C(v) = v up to rounding
        eng.close()


@pytest.mark.parametrize("rows,c", [(96, 16), (128, 64)])
def test_rank_k_levels_on_degenerate_matrices(rows, c):
    """Rank-K levels on arguments that stress the eigen-decomposition: a matrix of exact rank two (a singular
    Gram matrix; every level of rank two or more then recovers it: its entries are non-zero integers, so the
    rounded message is the matrix itself), magnitudes near both ends of the fp32 range, a zero vector (the
    node keeps its estimator), columns and rows a million times smaller than the rest.  (Entries that are
    exactly zero are left out on purpose: what a decomposition leaves there is rounding noise of its own,
    not comparable bit for bit.)"""
    E = _eng()
    d = rows * c
    rng = np.random.default_rng(7 * rows + c)
    wl = [(O.RANK, (1, c)), (O.RANK, (3, c)), (O.RANK, (c // 2, c)), (O.TOPK, d)]

    def structured():
        X = (rng.standard_normal((rows, 4)) * np.array([8.0, 4.0, 2.0, 1.0])) @ rng.standard_normal((4, c))
        return X + 0.3 * rng.standard_normal((rows, c))

    sign = lambda m: rng.choice([-1.0, 1.0], m)
    low = (4.0 * np.outer(sign(rows) * rng.integers(1, 4, rows), sign(c) * rng.integers(1, 4, c))
           + np.outer(sign(rows) * rng.choice([1.0, 3.0], rows), sign(c) * rng.choice([1.0, 3.0], c)))     # 4 a b + odd: never zero
    skewed = structured()
    skewed[:, 3] *= 1e-6
    skewed[:, c - 1] *= 1e-6
    skewed[rows // 2:, :] *= 1e-6
    cases = [low, structured() * 1e-18, structured() * 1e15, np.zeros((rows, c)), skewed]
    n = len(cases)
    v = np.stack([m.reshape(d) for m in cases]).astype(np.float32)
    assert np.linalg.matrix_rank(low) == 2 and np.all(low != 0)
    x0 = np.zeros(d, dtype=np.float32)
    for zeta, scale in ((1.0, 1e-9), (1.0, 0.05)):
        kw = dict(n=n, d=d, gamma=0.05, worker_levels=wl, zeta_worker=zeta, master_levels=[], zeta_master=0.0)
        orc = O.AdaCGDOracle(**kw)
        orc.init(x0, None, O.INIT_ZERO)
        eng = E.AdaCGD(grad_mode=E.DIFF_EXTERNAL, init_mode=E.INIT_ZERO, x0=_cuda(x0), flags=E.FLAG_ANY_LEVEL_ORDER, **kw)
        Dt = np.sum(v.astype(np.float64) ** 2, axis=1) * scale
        res, rm = orc.step(diffs=v, D=Dt)
        eng.step(_cuda(v), _cuda(Dt))
        vmax = np.abs(v).max(axis=1)
        with until_near_tie(("rank degenerate", rows, c, scale)):
            compare_step_rank(eng, orc, res, None, ("rank degenerate", rows, c, scale), vmax)
        lev = eng.state(E.F_LEVEL)
        assert lev[3] == 0                                   # the zero vector: nothing to send
        if scale == 1e-9:
            assert lev[0] == 2                               # exact rank two: the first level of rank >= 2 reproduces it
            assert np.array_equal(eng.state(E.F_GI)[0], v[0])
        assert np.isfinite(eng.state(E.F_RANK_SPECTRUM)).all() and np.isfinite(eng.state(E.F_GI)).all()
        eng.close()
