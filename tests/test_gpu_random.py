"""Randomised parity sweep: shapes around every tiling boundary, random level sets (Top-K sizes over four
decades, quantisers, the identity), trigger constants or per-position trigger pairs, the three ways to
start the estimators, input kinds and kernel paths, three steps each,
compared with the oracle bit for bit exactly as the fixed cases are."""
import numpy as np
import pytest

from oracle import adacgd_oracle as O
from test_gpu_parity import NearTie, _cuda, _eng, compare_step, make_vectors

pytestmark = pytest.mark.gpu

DIMS = [1, 2, 3, 63, 64, 65, 255, 1000, 2047, 2048, 2049, 4095, 4096, 4097, 8191, 8192, 8193, 20000,
        3 * 8192 + 516, 128 * 8192, 128 * 8192 + 4, 129 * 8192 + 2052, 131 * 8192 + 8188]


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_configurations_bit_exact(seed):
    _sweep(seed, 100, False)


@pytest.mark.parametrize("seed", [21, 22])
def test_random_configurations_with_block_wise_quantisers_bit_exact(seed):
    """The same sweep with block-wise quantiser levels (one scale per 64 ... 2048 coordinates) in most level sets."""
    _sweep(seed, 60, True)


def _sweep(seed, cases, with_blocks):
    E = _eng()
    rng = np.random.default_rng(seed)
    near_ties = 0
    for case in range(cases):
        d = int(rng.choice(DIMS))
        n = int(rng.integers(1, 3)) if d > 100000 else int(rng.integers(1, 7))
        Ks = sorted({int(max(1, min(d, round(d * 10 ** rng.uniform(-4, -0.3))))) for _ in range(int(rng.integers(1, 5)))})
        levels = [(O.TOPK, k) for k in Ks]
        if rng.random() < 0.4:
            for b in rng.choice([2, 3, 4, 6, 8], size=int(rng.integers(1, 3)), replace=False):
                levels.append((O.QUANT, int(b)))
        if with_blocks and rng.random() < 0.8:
            for _ in range(int(rng.integers(1, 3))):
                levels.append((O.QUANT_BLOCK, (int(rng.choice([2, 3, 4, 8])), int(rng.choice([64, 128, 256, 1024, 2048])))))
        if rng.random() < 0.3:
            levels.append((O.TOPK, d))
        levels = sorted(set(levels), key=lambda l: (O.level_alpha(l, d), l[0], str(l[1])))
        ml = [] if rng.random() < 0.2 else [(O.TOPK, int(max(1, min(d, round(d * 10 ** rng.uniform(-3, -0.5))))))]
        zw = float(rng.choice([0.0, 0.3, 1.0, 3.0]))
        zm = float(rng.choice([0.0, 0.0, 0.5]))
        kind = str(rng.choice(["normal", "ties", "heavy", "sparse", "const", "denormal"]))
        flags = int(rng.choice([0, 0, E.FLAG_TWO_PASS]))
        pseed = int(rng.integers(1, 2 ** 40))
        steps = 2 if d > 100000 else 3
        tag = (seed, case, n, d, levels, ml, zw, zm, kind, flags)
        grads = [make_vectors(rng, n, d, kind) for _ in range(steps + 1)]
        for t in range(1, steps + 1):
            grads[t] = (grads[t - 1] + grads[t] * np.float32(10.0 ** rng.uniform(-2, 0))).astype(np.float32)
        x0 = rng.standard_normal(d).astype(np.float32)
        diff_mode = rng.random() < 0.3       # the caller supplies x - h and ||x - y||^2 itself
        # a third of the cases: a (zeta_j, eta_j) pair per cascade position instead of the one constant
        tw = tm = None
        if rng.random() < 0.35:
            tw = [(float(rng.choice([0.0, 0.4, 1.0, 2.5])), float(rng.choice([0.0, 0.0, 0.05, 0.3]))) for _ in levels]
            tm = [(float(rng.choice([0.0, 0.5])), float(rng.choice([0.0, 0.1]))) for _ in ml]
        compressed_start = (not diff_mode) and levels[-1][0] == O.TOPK and rng.random() < 0.25
        kw = dict(n=n, d=d, gamma=0.05, worker_levels=levels, zeta_worker=zw, master_levels=ml, zeta_master=zm,
                  seed=pseed, worker_triggers=tw, master_triggers=tm)
        tag = tag + (tw, tm, diff_mode, compressed_start)
        orc = O.AdaCGDOracle(**kw)
        if diff_mode:
            orc.init(x0, None, O.INIT_ZERO)
            eng = E.AdaCGD(grad_mode=E.DIFF_EXTERNAL, init_mode=E.INIT_ZERO, x0=_cuda(x0), flags=flags, **kw)
        else:
            orc.init(x0, grads[0], O.INIT_COMPRESSED if compressed_start else O.INIT_FULLGRAD)
            eng = E.AdaCGD(grad_mode=E.GRAD_EXTERNAL, x0=_cuda(x0), grad0=_cuda(grads[0]), flags=flags,
                           init_mode=E.INIT_COMPRESSED if compressed_start else E.INIT_FULLGRAD, **kw)
        try:
            for t in range(1, steps + 1):
                if diff_mode:
                    Dt = np.sum(grads[t].astype(np.float64) ** 2, axis=1) * 10.0 ** rng.uniform(-2, 1, n)
                    res, rm = orc.step(diffs=grads[t], D=Dt)
                    eng.step(_cuda(grads[t]), _cuda(Dt))
                else:
                    res, rm = orc.step(grads=grads[t])
                    eng.step(_cuda(grads[t]))
                compare_step(eng, orc, res, rm, tag + (t,))
        except NearTie:
            near_ties += 1          # either decision is correct there: the rest of the case is left out, not the test
        finally:
            eng.close()
    assert near_ties <= 5
