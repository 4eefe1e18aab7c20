"""Experiment harness in the shape of the paper's Section 6 / Appendix "Experimental details":
GD, LAG, EF21 (Top-1), CLAG (Top-1) and AdaCGD on logistic regression with the nonconvex
regulariser, each run with multiples 2^0 .. 2^8 of its theoretical stepsize, stopped by the
communication cost, and compared by the squared norm of the full gradient.

All methods are special cases of the AdaCGD compressor (Section 4.3): one level = CLAG,
zeta = 0 = EF21, the identity level = LAG / GD, and run through the same engine.  The master
compressor is the identity here, as in the paper's experiments.

The datasets of the paper are not available; the seeded synthetic stand-ins of
`workloads.py` take their place.  The smoothness constants are computed on the host with
NumPy; every step of the method itself runs on the GPU.

Theoretical stepsize (nonconvex theorem for Ada3PC): gamma = 1 / (L_- + L_+ sqrt(B / A)),
with (A, B) the 3PC constants of the compressor.  The paper takes the constants of its
building blocks from the 3PC framework it extends; they are restated in `three_pc_constants`.
"""
import argparse
import math

import numpy as np

from . import workloads as W

METHODS = ("gd", "lag", "ef21", "clag", "adacgd")


def smoothness_constants(wl):
    """(L_minus, L_plus) of the Section 6 objective for a LogisticWorkload.

    The logistic term of f_i has Hessian <= A_i^T A_i / (4 N_i); the regulariser
    lambda x^2 / (1 + x^2) has second derivative in [-lambda/2, 2 lambda].  L_- bounds the
    smoothness of the average f, L_+^2 is the average of the squared constants of the f_i."""
    n = wl.n
    off = wl.shard_offsets
    A = wl.A.astype(np.float64)
    Li = []
    for i in range(n):
        Ai = A[off[i]:off[i + 1]]
        Li.append(np.linalg.eigvalsh(Ai.T @ Ai)[-1] / (4.0 * Ai.shape[0]) + 2.0 * wl.lam)
    # every f_i carries the full regulariser and f is their plain average
    rows = [off[i + 1] - off[i] for i in range(n)]
    H = sum((A[off[i]:off[i + 1]].T @ A[off[i]:off[i + 1]]) / (4.0 * rows[i]) for i in range(n)) / n
    L_minus = np.linalg.eigvalsh(H)[-1] + 2.0 * wl.lam
    L_plus = math.sqrt(float(np.mean(np.square(Li))))
    return float(L_minus), float(L_plus)


def ef21_constants(alpha):
    """3PC constants of the EF21 compressor built on an alpha-contractive compressor."""
    if alpha >= 1.0:
        return 1.0, 0.0
    r = math.sqrt(1.0 - alpha)
    return 1.0 - r, (1.0 - alpha) / (1.0 - r)


def three_pc_constants(method, alphas=(), zeta=0.0):
    """(A, B) with E||C_{h,y}(x) - x||^2 <= (1 - A) ||h - y||^2 + B ||x - y||^2.

    gd: exact (A = 1, B = 0).  lag: A = 1, B = zeta.  ef21: from the contraction parameter.
    clag: EF21's A, B = max(EF21's B, zeta).  adacgd: the minimum A and maximum B over its
    levels (Lemma 2 of the paper), each level being EF21 under a trigger, plus the LAG skip."""
    if method == "gd":
        return 1.0, 0.0
    if method == "lag":
        return 1.0, float(zeta)
    if method == "ef21":
        return ef21_constants(alphas[0])
    if method == "clag":
        a, b = ef21_constants(alphas[0])
        return a, max(b, float(zeta))
    if method == "adacgd":
        ab = [ef21_constants(a) for a in alphas]
        return min(a for a, _ in ab), max(max(b for _, b in ab), float(zeta))
    raise ValueError(method)


def theoretical_stepsize(L_minus, L_plus, A, B):
    return 1.0 / (L_minus + L_plus * math.sqrt(B / A))


def method_levels(method, d, adacgd_ratios=(0.01, 0.05, 0.1, 0.25, 0.5), zeta=1.0):
    """Level set and trigger constant that make the AdaCGD compressor equal to `method`.
    AdaCGD itself: Top-K levels from strong compression up to half of the coordinates."""
    if method == "gd":
        return [(W.TOPK, d)], 0.0
    if method == "lag":
        return [(W.TOPK, d)], zeta
    if method == "ef21":
        return [(W.TOPK, 1)], 0.0
    if method == "clag":
        return [(W.TOPK, 1)], zeta
    if method == "adacgd":
        Ks = sorted({W.ratio_K(r, d) for r in adacgd_ratios})
        return [(W.TOPK, k) for k in Ks], zeta
    raise ValueError(method)


def largest_message_bits(levels, d):
    """Cost of the most expensive message of a level set, by the rule of the engine's counters:
    level id + K (32 + ceil(log2 d)) bits for Top-K, + d b + 32 for b bits."""
    idb = max(1, math.ceil(math.log2(len(levels) + 1)))
    ib = max(1, math.ceil(math.log2(d)))
    return idb + max(p * (32 + ib) if kind == W.TOPK else d * p + 32 for kind, p in levels)


def run(wl, method, multiplier, bit_budget, max_steps=100000, zeta=1.0, chunk=50, base_gamma=None):
    """Runs one method on the GPU until the uplink cost reaches `bit_budget` bits per worker.
    Returns (steps, bits per worker, ||grad f(x)||^2), sampled after at most `chunk` steps: the
    number of steps between two samples is what the remaining budget covers at the price of the
    level set's most expensive message, so a run ends within one step of the budget."""
    import torch
    from . import engine as E
    levels, z = method_levels(method, wl.d, zeta=zeta)
    if base_gamma is None:
        Lm, Lp = smoothness_constants(wl)
        A_, B_ = three_pc_constants(method, [k / wl.d for _, k in levels], z)
        base_gamma = theoretical_stepsize(Lm, Lp, A_, B_)
    A, labels = torch.from_numpy(wl.A).cuda(), torch.from_numpy(wl.labels).cuda()
    x0 = torch.zeros(wl.d, dtype=torch.float32, device="cuda")
    eng = E.AdaCGD(n=wl.n, d=wl.d, gamma=base_gamma * multiplier, lam=wl.lam, worker_levels=levels,
                   zeta_worker=z, master_levels=[], zeta_master=0.0, grad_mode=E.GRAD_LOGISTIC, A=A,
                   labels=labels, shard_offsets=wl.shard_offsets, x0=x0)
    steps, bits, gn = [0], [0.0], []
    g = eng.state(E.F_PREV_GRAD).astype(np.float64).mean(axis=0)
    gn.append(float(g @ g))
    t = 0
    worst = largest_message_bits(levels, wl.d)
    while t < max_steps and bits[-1] < bit_budget and np.isfinite(gn[-1]):
        todo = int(min(chunk, max(1.0, (bit_budget - bits[-1]) / worst)))
        todo = min(todo, max_steps - t)
        eng.step(nsteps=todo)
        t += todo
        comm = eng.state(E.F_COMM)
        g = eng.state(E.F_PREV_GRAD).astype(np.float64).mean(axis=0)
        steps.append(t)
        bits.append(float(comm[1]) / wl.n)
        gn.append(float(g @ g))
    eng.close()
    return np.array(steps), np.array(bits), np.array(gn)


def sweep(wl, methods=METHODS, multipliers=tuple(2 ** k for k in range(9)), bit_budget=2e6, **kw):
    """For every method: the multiplier that reaches the lowest gradient norm within the budget."""
    Lm, Lp = smoothness_constants(wl)
    out = {}
    for m in methods:
        levels, z = method_levels(m, wl.d, zeta=kw.get("zeta", 1.0))
        A_, B_ = three_pc_constants(m, [k / wl.d for _, k in levels], z)
        g0 = theoretical_stepsize(Lm, Lp, A_, B_)
        best = None
        for mult in multipliers:
            s, b, gn = run(wl, m, mult, bit_budget, base_gamma=g0, **kw)
            final = gn[-1] if np.isfinite(gn[-1]) else float("inf")
            if best is None or final < best["grad_norm_sq"]:
                best = {"multiplier": mult, "grad_norm_sq": final, "steps": int(s[-1]), "bits_per_worker": float(b[-1]),
                        "gamma": g0 * mult, "curve": (s, b, gn)}
        out[m] = best
    return out


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--workload", choices=["tiny", "sparse_logreg"], default="sparse_logreg")
    ap.add_argument("--budget-bits", type=float, default=2e6, help="uplink bits per worker at which a run stops")
    ap.add_argument("--max-multiplier-log2", type=int, default=8)
    ap.add_argument("--zeta", type=float, default=1.0)
    ap.add_argument("--curves", metavar="FILE", help="write the best run of every method as CSV rows "
                    "method,step,bits_per_worker,grad_norm_sq (the axes of the paper's figures)")
    args = ap.parse_args()
    wl = W.tiny() if args.workload == "tiny" else W.sparse_logreg()
    res = sweep(wl, multipliers=tuple(2 ** k for k in range(args.max_multiplier_log2 + 1)),
                bit_budget=args.budget_bits, zeta=args.zeta)
    print("%-8s %10s %12s %10s %16s %14s" % ("method", "multiplier", "gamma", "steps", "bits/worker", "|grad f|^2"))
    for m, r in res.items():
        print("%-8s %10d %12.4g %10d %16.4g %14.6g" % (m, r["multiplier"], r["gamma"], r["steps"],
                                                     r["bits_per_worker"], r["grad_norm_sq"]))
    if args.curves:
        with open(args.curves, "w") as f:
            f.write("method,step,bits_per_worker,grad_norm_sq\n")
            for m, r in res.items():
                for st, b, g in zip(*r["curve"]):
                    f.write("%s,%d,%.17g,%.17g\n" % (m, st, b, g))


if __name__ == "__main__":
    main()
