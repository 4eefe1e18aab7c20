#!/usr/bin/env python3
"""Benchmark of the AdaCGD hot path on one MI355X.

A step is one full iteration of Algorithm 2 on the model-sized workload (n = 16
workers, d = 11.2 M, Top-K levels at {1e-4, 1e-3, 1e-2, 5e-2} d, master Top-K at
1e-2 d): iterate update, worker compression with level choice for all workers,
server aggregation, master compression.  The per-worker gradients are supplied
(seeded synthetic vectors already resident in HBM), as that workload defines them.

Prints one JSON line: throughput (compressed floats per second = n d steps / s)
of the whole step on ONE stream -- every kernel of step t finishes before step
t+1 starts, as the data dependence of Algorithm 1 demands when gradients are
computed at the new iterate --, the two-stream figure beside it, the roofline
position of the worker compression kernels from HIP-event timings taken inside the
library, a sweep over the trigger constant zeta, the CPU oracle timed on the same
inputs (one core, then all cores), and the secondary workloads.
"""
import argparse
import concurrent.futures as cf
import hashlib
import json
import multiprocessing as mp
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# Vector-ALU issue peak: 256 compute units x 4 SIMDs, one 64-lane instruction every 4 cycles at 2.4 GHz
# = 39.3e12 lane-instructions per second (the 157.3 TFLOP/s fp32 figure is this x 2 flops per FMA x 2 for
# packed operations).
VALU_PEAK_LANE_INSTS = 256 * 4 * 64 * 2.4e9 / 4
ZETAS = (0.0, 0.25, 1.0, 4.0, 16.0)
COUNTERS_JSON = os.path.join(ROOT, "profiles", "counters.json")
CSRC = os.path.join(ROOT, "paper_2211_00188_amd", "csrc")


def kernel_sources_digest():
    """sha256 over the kernel sources: counter figures are only valid for the code they were taken on."""
    h = hashlib.sha256()
    for fn in sorted(os.listdir(CSRC)):
        if fn.endswith((".hip", ".h")):
            h.update(fn.encode())
            h.update(open(os.path.join(CSRC, fn), "rb").read())
    return h.hexdigest()


def load_counters():
    """Figures taken from rocprofv3 --pmc runs (profiles/counters.json, written next to the summaries under
    profiles/), or {} if the kernel sources have changed since: nothing measured is then claimed."""
    try:
        rec = json.load(open(COUNTERS_JSON))
    except (OSError, ValueError):
        return {}
    return rec if rec.get("csrc_sha256") == kernel_sources_digest() else {}


# ---------------------------------------------------------------------------------------------------
# CPU oracle on the benchmark's inputs (runs before the GPU is touched: worker processes are forked)
# ---------------------------------------------------------------------------------------------------
_CPU = {}


def _cpu_worker(i):
    from oracle import adacgd_oracle as O
    g0, g1, levels, zeta = _CPU["g0"], _CPU["g1"], _CPU["levels"], _CPU["zeta"]
    r = O.adacgd_compress(g0[i], g0[i], g1[i], levels, zeta)
    return r.level, r.msg_idx, r.msg_val


def _cpu_server(results, gt0, n, d, master_levels):
    from oracle import adacgd_oracle as O
    acc = np.zeros(d, dtype=np.float64)
    for level, idx, val in results:
        if level > 0:
            acc[idx] += val.astype(np.float64)
    gt1 = (gt0.astype(np.float64) + acc / n).astype(np.float32)
    O.adacgd_compress(gt0, gt0, gt1, master_levels, 0.0)


def cpu_baseline(wk, g0, g1):
    """One whole step of the oracle (all n worker compressions with every level and the level choice,
    server aggregation, master compression) on the first two gradient arrays of the workload: on one
    core, then with one process per worker on the cores this job may use."""
    n, d = wk.n, wk.d
    _CPU.update(g0=g0, g1=g1, levels=wk.worker_levels, zeta=wk.zeta_worker)
    gt0 = (g0.astype(np.float64).sum(axis=0) / n).astype(np.float32)
    t0 = time.perf_counter()
    res = [_cpu_worker(i) for i in range(n)]
    _cpu_server(res, gt0, n, d, wk.master_levels)
    t_one = time.perf_counter() - t0
    cores = len(os.sched_getaffinity(0))
    procs = max(1, min(n, cores))
    t0 = time.perf_counter()
    with cf.ProcessPoolExecutor(max_workers=procs, mp_context=mp.get_context("fork")) as ex:
        res = list(ex.map(_cpu_worker, range(n)))
    _cpu_server(res, gt0, n, d, wk.master_levels)
    t_all = time.perf_counter() - t0
    _CPU.clear()
    what = ("one whole oracle step (compression of all %d workers with every level and the level choice, "
            "server aggregation, master compression) at d=%d on the benchmark's first two gradient arrays" % (n, d))
    return {"value": n * d / t_all, "unit": "floats/s", "cores": procs, "kind": "oracle",
            "sample": what + "; one process per worker on the %d cores of this job (cores available: %d)" % (procs, cores),
            "seconds": t_all,
            "single_core": {"value": n * d / t_one, "unit": "floats/s", "cores": 1, "seconds": t_one}}


# ---------------------------------------------------------------------------------------------------
# secondary workloads
# ---------------------------------------------------------------------------------------------------
def _timed_steps(eng, E, torch, step_fn, warmup, steps):
    for t in range(warmup):
        step_fn(t)
    torch.cuda.synchronize()
    eng.kernel_ms()
    h0 = eng.state(E.F_LEVEL_HIST).astype(np.int64)
    t0 = time.perf_counter()
    for t in range(warmup, warmup + steps):
        step_fn(t)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    hist = eng.state(E.F_LEVEL_HIST).astype(np.int64) - h0
    kms = {k: round(ms / cnt, 5) for k, (ms, cnt) in eng.kernel_ms().items() if cnt}
    return dt, hist, kms


def _message_bytes(levels, hist, d, steps):
    """Algorithmic bytes per step for what the chosen levels send and update: a Top-K entry is 8 B of
    message + 4 B of estimator written; a b-bit level reads and writes the estimator (8 B) and writes a
    code of b bits per coordinate."""
    total = 0.0
    for j in range(1, len(hist)):
        kind, param = levels[j - 1]
        total += float(hist[j]) * (12.0 * param if kind == 0 else d * (8.0 + param / 8.0))
    return total / steps


def _two_ceilings(kms, group, alg_bytes, coords, counters):
    """Roofline entry of a compression step whose level set holds quantisers: the HBM ceiling on the
    algorithmic bytes and the vector-ALU ceiling on the instructions the counters show, per kernel of the
    group and for the group as a whole."""
    group = [k for k in group if k in kms]
    t = sum(kms[k] for k in group) * 1e-3
    insts = (counters or {}).get("valu_lane_insts_per_worker_coordinate", {})
    busy = (counters or {}).get("valu_busy", {})
    have = all(k in insts for k in group)
    total_insts = sum(insts[k] for k in group) * coords if have else None
    hbm = {"achieved": alg_bytes / t / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": alg_bytes / t / 1e9 / HBM_PEAK_GBS}
    alu = None
    if have:
        alu = {"achieved": total_insts / t, "peak": VALU_PEAK_LANE_INSTS, "unit": "lane-instructions/s",
               "frac": total_insts / t / VALU_PEAK_LANE_INSTS}
    per_kernel = {}
    for k in group:
        per_kernel[k] = {"avg_ms": kms[k],
                         "valu_lane_insts_per_worker_coordinate": insts.get(k),
                         "alu_frac": insts[k] * coords / (kms[k] * 1e-3) / VALU_PEAK_LANE_INSTS if k in insts else None,
                         "valu_busy_from_counters": busy.get(k)}
    bound = "alu" if (alu and alu["frac"] > hbm["frac"]) else "hbm"
    main = alu if bound == "alu" else hbm
    return {"bound": bound, "kernel": "+".join(group), "achieved": main["achieved"], "peak": main["peak"],
            "unit": main["unit"], "frac": main["frac"], "traffic": None, "avg_ms_per_step": t * 1e3,
            "algorithmic_bytes_per_step": alg_bytes, "hbm_ceiling": hbm, "alu_ceiling": alu, "kernels": per_kernel,
            "counters": "profiles/counters.json" if have else None}


def extra_kernel_stress(E, W, torch, counters, steps=50, warmup=4):
    """Secondary workload: heavy-tailed difference vectors, mixed Top-K / b-bit level set (n=32, d=2^20)."""
    wk = W.kernel_stress()
    pool = [W.kernel_stress_diffs(wk, t) for t in range(4)]
    dv = [(torch.from_numpy(v).cuda(), torch.from_numpy(D).cuda()) for v, D in pool]
    x0 = torch.zeros(wk.d, dtype=torch.float32, device="cuda")
    eng = E.AdaCGD(n=wk.n, d=wk.d, gamma=0.1, worker_levels=wk.worker_levels, zeta_worker=wk.zeta_worker,
                   master_levels=wk.master_levels, zeta_master=0.0, grad_mode=E.DIFF_EXTERNAL,
                   init_mode=E.INIT_ZERO, x0=x0, seed=wk.seed, flags=E.FLAG_KERNEL_TIMING)
    dt, hist, kms = _timed_steps(eng, E, torch, lambda t: eng.step(*dv[t % 4]), warmup, steps)
    eng.close()
    # difference mode: the step reads v once (4 B per worker-coordinate) plus what the chosen levels move
    alg = 4.0 * wk.n * wk.d + _message_bytes(wk.worker_levels, hist, wk.d, steps)
    group = ["w_scan", "w_filter", "w_gather", "w_select", "w_tally", "w_compact", "w_qapply"]
    return {"workload": "kernel stress: n=%d, d=%d, difference vectors exp(N(0,1)) * t3, levels %s, master Top-%d"
                        % (wk.n, wk.d, wk.worker_levels, wk.master_levels[0][1]),
            "steps": steps, "ms_per_step": dt / steps * 1e3, "floats_per_sec": wk.n * wk.d * steps / dt,
            "zeta_worker": wk.zeta_worker,
            "level_histogram_skip_then_levels": [int(v) for v in hist], "kernels_avg_ms": kms,
            "roofline": _two_ceilings(kms, group, alg, wk.n * wk.d, counters.get("kernel_stress")),
            "note": "one stream, HIP events around every kernel; each n x d array (134 MB) fits the 256 MB "
                    "memory-side cache, so HBM traffic is below the algorithmic bytes"}


def extra_block_quant(E, W, torch, counters, steps=50, warmup=4):
    """Secondary workload: the kernel-stress vectors with block-wise quantiser levels (one scale per 256 coordinates)."""
    wk = W.kernel_stress_blockwise()
    pool = [W.kernel_stress_diffs(wk, t) for t in range(4)]
    dv = [(torch.from_numpy(v).cuda(), torch.from_numpy(D).cuda()) for v, D in pool]
    x0 = torch.zeros(wk.d, dtype=torch.float32, device="cuda")
    eng = E.AdaCGD(n=wk.n, d=wk.d, gamma=0.1, worker_levels=wk.worker_levels, zeta_worker=wk.zeta_worker,
                   master_levels=wk.master_levels, zeta_master=0.0, grad_mode=E.DIFF_EXTERNAL,
                   init_mode=E.INIT_ZERO, x0=x0, seed=wk.seed, flags=E.FLAG_KERNEL_TIMING)
    dt, hist, kms = _timed_steps(eng, E, torch, lambda t: eng.step(*dv[t % 4]), warmup, steps)
    eng.close()
    sent = 0.0
    for j in range(1, len(hist)):
        kind, param = wk.worker_levels[j - 1]
        sent += float(hist[j]) * (12.0 * param if kind == 0 else wk.d * (8.0 + param[0] / 8.0) + 4.0 * wk.d / param[1])
    alg = 4.0 * wk.n * wk.d + sent / steps
    group = ["w_scan", "w_filter", "w_gather", "w_select", "w_tally", "w_compact", "w_qapply"]
    return {"workload": "kernel stress with block-wise quantisers: n=%d, d=%d, levels %s, master Top-%d"
                        % (wk.n, wk.d, wk.worker_levels, wk.master_levels[0][1]),
            "steps": steps, "ms_per_step": dt / steps * 1e3, "floats_per_sec": wk.n * wk.d * steps / dt,
            "zeta_worker": wk.zeta_worker,
            "level_histogram_skip_then_levels": [int(v) for v in hist], "kernels_avg_ms": kms,
            "roofline": _two_ceilings(kms, group, alg, wk.n * wk.d, counters.get("block_quant")),
            "note": "one stream, HIP events around every kernel"}


def extra_rank_k(E, W, torch, steps=20, warmup=3):
    """Secondary workload: matrix-shaped gradients (16384 x 64 per worker) with Rank-K levels."""
    wk = W.matrix_shaped()
    gen = W.MatrixShapedGrads(wk)
    g0 = torch.from_numpy(gen.next()).cuda()
    pool = [torch.from_numpy(gen.next()).cuda() for _ in range(4)]
    x0 = torch.zeros(wk.d, dtype=torch.float32, device="cuda")
    eng = E.AdaCGD(n=wk.n, d=wk.d, gamma=0.1, worker_levels=wk.worker_levels, zeta_worker=wk.zeta_worker,
                   master_levels=wk.master_levels, zeta_master=0.0, grad_mode=E.GRAD_EXTERNAL,
                   init_mode=E.INIT_FULLGRAD, x0=x0, grad0=g0, flags=E.FLAG_KERNEL_TIMING | E.FLAG_RETAIN_EXT)
    for t in range(warmup):
        eng.step(pool[t % 4])
    torch.cuda.synchronize()
    eng.kernel_ms()
    h0 = eng.state(E.F_LEVEL_HIST).astype(np.int64)
    t0 = time.perf_counter()
    for t in range(warmup, warmup + steps):
        eng.step(pool[t % 4])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    hist = eng.state(E.F_LEVEL_HIST).astype(np.int64) - h0
    raw = eng.kernel_ms()
    eng.close()
    per_step = {k: round(ms / steps, 5) for k, (ms, cnt) in raw.items() if cnt}      # summed over the launches of a step
    c, rows = wk.cols, wk.rows
    ks = [prm[0] for k, prm in wk.worker_levels if k == W.RANK]
    active = float(hist[1:].sum()) / steps                      # workers per step that did not skip
    sent = [float(hist[j]) / steps if wk.worker_levels[j - 1][0] == W.RANK else 0.0 for j in range(1, len(hist))]
    # fp64 flops as issued to the matrix cores (16 x 16 x 4 instructions of 2048 flops).  Per 16 rows of X:
    # the Gram matrix takes 4 instructions for each of the nb (nb + 1) / 2 upper tiles (nb = c / 16); Y = X V
    # c / 4 for each block of 16 eigenvectors; X_K = Y V_K^T nb ceil(K / 4) per level.
    nb = c // 16
    kp = lambda kmax: (kmax + 15) // 16
    per16_gram = 4 * nb * (nb + 1) // 2
    per16_err = (c // 4) * kp(max(ks)) + sum(nb * ((k + 3) // 4) for k in ks)
    flops = 2048.0 * (rows / 16.0) * (active * (per16_gram + per16_err)
                                      + sum(sj * ((c // 4) * kp(wk.worker_levels[j][1][0]) + nb * ((wk.worker_levels[j][1][0] + 3) // 4))
                                            for j, sj in enumerate(sent) if sj))
    # algorithmic bytes: Gram and error kernels read x and the estimator (8 B per coordinate each); the update
    # reads both, writes the message and the estimator (16 B)
    nbytes = wk.d * (active * 16.0 + sum(sent) * 16.0)
    t_rank = per_step.get("w_rank", 0.0) * 1e-3
    t_eig = per_step.get("w_eig", 0.0) * 1e-3
    hbm = {"achieved": nbytes / t_rank / 1e9 if t_rank else None, "peak": HBM_PEAK_GBS, "unit": "GB/s",
           "frac": nbytes / t_rank / 1e9 / HBM_PEAK_GBS if t_rank else None}
    mfma = {"achieved": flops / t_rank / 1e12 if t_rank else None, "peak": 78.6, "unit": "TFLOP/s (fp64)",
            "frac": flops / t_rank / 1e12 / 78.6 if t_rank else None}
    bound = "hbm" if (hbm["frac"] or 0) >= (mfma["frac"] or 0) else "mfma"
    main = hbm if bound == "hbm" else mfma
    return {"workload": "matrix-shaped gradients: n=%d workers, %d x %d per worker (d=%d), shared directions + noise, "
                        "levels %s, master Top-%d" % (wk.n, wk.rows, wk.cols, wk.d, wk.worker_levels, wk.master_levels[0][1]),
            "steps": steps, "ms_per_step": dt / steps * 1e3, "floats_per_sec": wk.n * wk.d * steps / dt,
            "zeta_worker": wk.zeta_worker,
            "level_histogram_skip_then_levels": [int(v) for v in hist], "kernels_ms_per_step": per_step,
            "roofline": {"bound": bound, "kernel": "w_rank (Gram matrix, realised errors and update of the Rank-K levels)",
                         "achieved": main["achieved"], "peak": main["peak"], "unit": main["unit"], "frac": main["frac"],
                         "traffic": None, "ms_per_step": t_rank * 1e3, "algorithmic_bytes_per_step": nbytes,
                         "fp64_flops_per_step": flops, "hbm_ceiling": hbm, "mfma_ceiling": mfma},
            "eigen_decomposition": {"ms_per_step": t_eig * 1e3, "matrices_per_step": active, "size": c,
                                    "note": "one block per matrix (cyclic Jacobi in LDS): latency-bound, no roofline applies"},
            "note": "one stream, HIP events around every kernel"}


def extra_federated(E, W, torch, n, counters, steps=10, warmup=2):
    """Secondary workload: logistic-regression shards (engine computes the gradients), d=65536, 32 samples each."""
    wl = W.federated(n=n)
    A, labels = torch.from_numpy(wl.A).cuda(), torch.from_numpy(wl.labels).cuda()
    x0 = torch.zeros(wl.d, dtype=torch.float32, device="cuda")

    def engine(zeta, flags):
        return E.AdaCGD(n=wl.n, d=wl.d, gamma=wl.gamma, lam=wl.lam, worker_levels=wl.worker_levels,
                        zeta_worker=zeta, master_levels=wl.master_levels, zeta_master=wl.zeta_master,
                        grad_mode=E.GRAD_LOGISTIC, A=A, labels=labels, shard_offsets=wl.shard_offsets, x0=x0, seed=5,
                        flags=flags)

    eng = engine(wl.zeta_worker, E.FLAG_KERNEL_TIMING)
    dt, hist, kms = _timed_steps(eng, E, torch, lambda t: eng.step(), warmup, steps)
    eng.close()
    sweep = []
    for zeta in ZETAS:                   # every branch of the cascade: skips, sparse levels, dense levels
        eng = engine(zeta, 0)
        dz, hz, _ = _timed_steps(eng, E, torch, lambda t: eng.step(), warmup, steps)
        eng.close()
        sweep.append({"zeta_worker": zeta, "ms_per_step": dz / steps * 1e3,
                      "level_histogram_skip_then_levels": [int(v) for v in hz]})
    a_bytes = float(wl.A.nbytes)
    grad_ms = kms.get("grad_margin", 0.0) + kms.get("grad_cols", 0.0)
    alg = 12.0 * wl.n * wl.d + _message_bytes(wl.worker_levels, hist, wl.d, steps)
    group = ["w_scan", "w_filter", "w_gather", "w_select", "w_tally", "w_compact", "w_qapply"]
    return {"workload": "federated logistic regression: n=%d workers, d=%d, %d samples each, "
                        "levels %s, master Top-%d" % (wl.n, wl.d, wl.A.shape[0] // wl.n, wl.worker_levels,
                                                      wl.master_levels[0][1]),
            "steps": steps, "ms_per_step": dt / steps * 1e3, "floats_per_sec": wl.n * wl.d * steps / dt,
            "zeta_worker": wl.zeta_worker,
            "level_histogram_skip_then_levels": [int(v) for v in hist], "kernels_avg_ms": kms,
            "gradient_kernels": {"algorithmic_bytes": 2 * a_bytes, "avg_ms": grad_ms,
                                 "GB/s": 2 * a_bytes / (grad_ms * 1e-3) / 1e9 if grad_ms else None,
                                 "frac_of_8TBps": 2 * a_bytes / (grad_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if grad_ms else None},
            "roofline_compression_step": _two_ceilings(kms, group, alg, wl.n * wl.d,
                                                       counters.get("federated") if n == 1000 else None),
            "zeta_sweep": sweep,
            "note": "one stream; the first record has HIP events around every kernel, the sweep has none"}


def extra_sparse_features(E, W, torch, steps=20, warmup=3):
    """Secondary workload: logistic regression on binary features kept as compressed sparse rows."""
    wl = W.sparse_features()
    nnz = int(wl.csr[0][-1])
    rows = wl.labels.shape[0]
    x0 = torch.zeros(wl.d, dtype=torch.float32, device="cuda")
    labels = torch.from_numpy(wl.labels).cuda()

    def engine(zeta, flags):
        return E.AdaCGD(n=wl.n, d=wl.d, gamma=wl.gamma, lam=wl.lam, worker_levels=wl.worker_levels,
                        zeta_worker=zeta, master_levels=wl.master_levels, zeta_master=wl.zeta_master,
                        grad_mode=E.GRAD_LOGISTIC_CSR, labels=labels, shard_offsets=wl.shard_offsets, csr=wl.csr, x0=x0,
                        flags=flags)

    eng = engine(wl.zeta_worker, E.FLAG_KERNEL_TIMING)
    dt, hist, kms = _timed_steps(eng, E, torch, lambda t: eng.step(), warmup, steps)
    eng.close()
    sweep = []
    for zeta in (0.0, 1.0, 4.0, 16.0, 64.0, 256.0):      # up to where every worker keeps its estimator in most steps
        eng = engine(zeta, 0)
        dz, hz, _ = _timed_steps(eng, E, torch, lambda t: eng.step(), warmup, steps)
        eng.close()
        sweep.append({"zeta_worker": zeta, "ms_per_step": dz / steps * 1e3,
                      "level_histogram_skip_then_levels": [int(v) for v in hz]})
    # stored entries: column + gathered x (margins), row + gathered fp64 margin (column sums); per row the
    # pointer, label and margin; per (worker, column) the column pointer and the gradient written
    alg = nnz * (4 + 4 + 4 + 8) + rows * (8 + 4 + 8) + wl.n * wl.d * (4 + 4)
    grad_ms = kms.get("grad_margin", 0.0) + kms.get("grad_cols", 0.0)
    return {"workload": "sparse binary features: n=%d workers, d=%d, %d rows each, %d stored entries per row, "
                        "Top-K levels %s, master Top-%d" % (wl.n, wl.d, rows // wl.n, nnz // rows,
                                                            [k for _, k in wl.worker_levels], wl.master_levels[0][1]),
            "steps": steps, "ms_per_step": dt / steps * 1e3, "floats_per_sec": wl.n * wl.d * steps / dt,
            "zeta_worker": wl.zeta_worker,
            "level_histogram_skip_then_levels": [int(v) for v in hist], "kernels_avg_ms": kms,
            "gradient_kernels": {"algorithmic_bytes": alg, "avg_ms": grad_ms,
                                 "GB/s": alg / (grad_ms * 1e-3) / 1e9 if grad_ms else None,
                                 "dense_matrix_bytes_for_comparison": 4.0 * rows * wl.d},
            "zeta_sweep": sweep,
            "note": "one stream; the first record has HIP events around every kernel, the sweep has none"}


def extra_small_logistic(E, W, torch, wl, steps, sparse_rows=False):
    """Launch-bound small configurations: steps per second and kernel launches per step only."""
    labels = torch.from_numpy(wl.labels).cuda()
    x0 = torch.zeros(wl.d, dtype=torch.float32, device="cuda")
    kw = dict(n=wl.n, d=wl.d, gamma=wl.gamma, lam=wl.lam, worker_levels=wl.worker_levels,
              zeta_worker=wl.zeta_worker, master_levels=wl.master_levels, zeta_master=wl.zeta_master,
              labels=labels, shard_offsets=wl.shard_offsets, x0=x0)
    if sparse_rows:
        kw.update(grad_mode=E.GRAD_LOGISTIC_CSR, csr=W.to_csr(wl.A, binary=True))
    else:
        kw.update(grad_mode=E.GRAD_LOGISTIC, A=torch.from_numpy(wl.A).cuda())
    eng = E.AdaCGD(flags=0, **kw)
    eng.step(nsteps=500)                   # a step takes tens of microseconds: let the clocks settle
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    eng.step(nsteps=steps)                 # one call enqueues all steps: no Python in the loop
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    hist = eng.state(E.F_LEVEL_HIST).astype(np.int64)
    eng.close()
    eng = E.AdaCGD(flags=E.FLAG_KERNEL_TIMING, **kw)     # second engine only to count the launches of a step
    eng.step(nsteps=5)
    torch.cuda.synchronize()
    km = eng.kernel_ms()                   # one timed slot per launch, except select (two launches per slot)
    launches = (sum(cnt for _, cnt in km.values()) + km["w_select"][1] + km["m_select"][1]) / 5.0
    eng.close()
    return {"workload": "%s%s: n=%d, d=%d, %d samples each, logistic regression, levels %s"
                        % (wl.name, " (features as sparse rows)" if sparse_rows else "", wl.n, wl.d,
                           wl.A.shape[0] // wl.n, [k for _, k in wl.worker_levels]),
            "steps": steps, "ms_per_step": dt / steps * 1e3, "steps_per_sec": steps / dt,
            "zeta_worker": wl.zeta_worker, "kernel_launches_per_step": launches,
            "level_histogram_skip_then_levels_since_init": [int(v) for v in hist],
            "note": "a step is four short dependent kernels: latency-bound, no roofline applies"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--repeats", type=int, default=5, help="timed regions of --steps steps each (median and min are reported)")
    ap.add_argument("--pool", type=int, default=4, help="distinct gradient arrays cycled through")
    ap.add_argument("--zeta", type=float, default=1.0)
    ap.add_argument("--n", type=int, default=16)
    ap.add_argument("--d", type=int, default=11_200_000)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the secondary workloads")
    ap.add_argument("--no-sweep", action="store_true", help="skip the zeta sweep of the main workload")
    ap.add_argument("--federated-n", type=int, default=1000,
                    help="workers of the secondary federated workload (1000 = the full configuration, 8.4 GB of features)")
    ap.add_argument("--secondary", choices=["kernel_stress", "federated", "sparse_features", "block_quant", "rank_k"],
                    help="run only this secondary workload and print its record (for profiling it on its own)")
    ap.add_argument("--no-overlap", action="store_true", help="skip the two-stream run")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: the engine runs on one GPU only (all n workers are batched on it); "
              "--gpus > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    from paper_2211_00188_amd import workloads as W
    counters = load_counters()

    wk = gen = host0 = None
    pool_host = []
    cpu = None
    if not args.secondary:
        wk = W.model_sized(n=args.n, d=args.d, zeta=args.zeta)
        gen = W.ModelSizedGrads(wk)
        host0 = gen.next().copy()
        pool_host = [gen.next().copy() for _ in range(args.pool)]
        if not args.no_cpu_baseline:
            cpu = cpu_baseline(wk, host0, pool_host[0])      # before the GPU is initialised: it forks

    import torch
    from paper_2211_00188_amd import engine as E

    torch.cuda.set_device(0)
    if args.secondary:
        rec = {"kernel_stress": lambda: extra_kernel_stress(E, W, torch, counters),
               "federated": lambda: extra_federated(E, W, torch, args.federated_n, counters),
               "sparse_features": lambda: extra_sparse_features(E, W, torch),
               "block_quant": lambda: extra_block_quant(E, W, torch, counters),
               "rank_k": lambda: extra_rank_k(E, W, torch)}[args.secondary]()
        print(json.dumps({"secondary_workload": rec}))
        return
    n, d = wk.n, wk.d
    g0 = torch.from_numpy(host0).cuda()
    pool = [torch.from_numpy(a).cuda() for a in pool_host]
    del host0, pool_host
    x0 = torch.zeros(d, dtype=torch.float32, device="cuda")

    repairs = []

    def run(flags, steps, warmup, repeats, zeta=None):
        """Returns the seconds of each of `repeats` timed regions of `steps` steps (each bracketed by a
        device synchronisation), the level histogram of the first region and the per-kernel timings."""
        eng = E.AdaCGD(n=n, d=d, gamma=0.1, worker_levels=wk.worker_levels,
                       zeta_worker=wk.zeta_worker if zeta is None else zeta,
                       master_levels=wk.master_levels, zeta_master=wk.zeta_master, grad_mode=E.GRAD_EXTERNAL,
                       init_mode=E.INIT_FULLGRAD, x0=x0, grad0=g0, flags=flags | E.FLAG_RETAIN_EXT)
        t = 0
        for _ in range(warmup):
            eng.step(pool[t % len(pool)])
            t += 1
        torch.cuda.synchronize()
        if flags & E.FLAG_KERNEL_TIMING:
            eng.kernel_ms()                 # drop the warm-up's timings
        h0 = eng.state(E.F_LEVEL_HIST).astype(np.int64)
        times, hist = [], None
        for _ in range(repeats):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                eng.step(pool[t % len(pool)])
                t += 1
            torch.cuda.synchronize()
            times.append(time.perf_counter() - t0)
            if hist is None:
                hist = eng.state(E.F_LEVEL_HIST).astype(np.int64) - h0
        kms = eng.kernel_ms() if flags & E.FLAG_KERNEL_TIMING else None
        repairs.append([int(v) for v in eng.state(E.F_REPAIRS)])
        cands = [int(v) for v in eng.state(E.F_CANDIDATES)]
        eng.close()
        del eng
        torch.cuda.empty_cache()
        return times, hist, kms, cands

    def stats(times, steps):
        ms = [t / steps * 1e3 for t in times]
        return {"first": ms[0], "median": statistics.median(ms), "min": min(ms), "all": [round(v, 5) for v in ms]}

    t_one, hist, _, cands = run(0, args.steps, args.warmup, args.repeats)
    one = stats(t_one, args.steps)
    two = None
    if not args.no_overlap:
        t_two, _, _, _ = run(E.FLAG_OVERLAP, args.steps, args.warmup, args.repeats)
        two = stats(t_two, args.steps)
    t_ev, hist_ev, kms, _ = run(E.FLAG_KERNEL_TIMING, args.steps, args.warmup, 1)

    sweep = []
    if not args.no_sweep:
        for zeta in ZETAS:
            tz, hz, _, _ = run(0, 8, 3, 1, zeta=zeta)
            sweep.append({"zeta_worker": zeta, "ms_per_step": tz[0] / 8 * 1e3,
                          "level_histogram_skip_then_levels": [int(v) for v in hz]})

    dt = statistics.median(t_one)          # a region of exactly --steps steps between two synchronisations: the median one
    steps_per_s = args.steps / dt
    floats_per_s = n * d * steps_per_s
    # algorithmic bytes of the worker compression step: one read of grad, g~_i, previous grad
    # (12 B per worker-coordinate) plus the message (8 B) and estimator write (4 B) per sent entry
    sent = sum(int(hist_ev[j]) * wk.worker_levels[j - 1][1] for j in range(1, len(hist_ev)))
    alg_bytes_step = 12.0 * n * d + 12.0 * sent / args.steps
    group = ["w_sample", "w_scan", "w_filter", "w_gather", "w_select", "w_tally", "w_compact"]
    per_kernel = {}
    for k, (ms, cnt) in kms.items():
        if cnt:
            per_kernel[k] = {"avg_ms": ms / cnt, "launches": cnt}
    group = [k for k in group if k in per_kernel]
    group_ms = sum(per_kernel[k]["avg_ms"] for k in group)
    achieved = alg_bytes_step / (group_ms * 1e-3) / 1e9
    dom = max(group, key=lambda k: per_kernel[k]["avg_ms"])
    dom_bytes = {"w_scan": 12.0 * n * d, "w_filter": 8.0 * n * d}.get(dom, 0.0)
    # HBM bytes of the same kernels from the FETCH_SIZE / WRITE_SIZE counter runs: only for the default
    # workload, the same kernel list, and kernel sources unchanged since the counters were taken
    default_workload = (args.n, args.d, args.zeta, args.pool) == (16, 11_200_000, 1.0, 4)
    tr = counters.get("model_sized", {})
    traffic = tr.get("traffic_bytes_per_step") if default_workload and tr.get("kernels") == "+".join(group) else None
    roofline = {
        "bound": "hbm", "kernel": "+".join(group), "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
        "traffic_GBps": traffic / (group_ms * 1e-3) / 1e9 if traffic else None,
        "traffic_source": tr.get("source") if traffic else None,
        "algorithmic_bytes_per_step": alg_bytes_step, "avg_ms_per_step": group_ms,
        "dominant_kernel": {"name": dom, "avg_ms": per_kernel[dom]["avg_ms"],
                            "bytes_read_per_launch": dom_bytes,
                            "GB/s": dom_bytes / (per_kernel[dom]["avg_ms"] * 1e-3) / 1e9,
                            "frac": dom_bytes / (per_kernel[dom]["avg_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "kernels_avg_ms": {k: round(v["avg_ms"], 5) for k, v in per_kernel.items()},
    }

    npool = len(pool)
    del pool, g0, x0
    torch.cuda.empty_cache()
    other = []
    if not args.no_extras:
        other.append(extra_kernel_stress(E, W, torch, counters))
        other.append(extra_block_quant(E, W, torch, counters))
        other.append(extra_rank_k(E, W, torch))
        other.append(extra_federated(E, W, torch, args.federated_n, counters))
        other.append(extra_small_logistic(E, W, torch, W.tiny(), 2000))
        other.append(extra_small_logistic(E, W, torch, W.sparse_logreg(), 2000))
        other.append(extra_small_logistic(E, W, torch, W.sparse_logreg(), 2000, sparse_rows=True))
        other.append(extra_sparse_features(E, W, torch))

    out = {
        "metric": "adacgd_compressed_floats_per_sec", "value": floats_per_s, "unit": "floats/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "steps_per_sec": steps_per_s,
        "ms_per_step_one_stream": one, "ms_per_step_two_streams": two,
        "value_two_streams": n * d / (two["median"] * 1e-3) if two else None,
        "config": {"workload": "model-sized vectors: n=%d workers, d=%d, external gradients "
                               "(shared AR(1) drift + 0.5 * per-worker offset), Top-K levels %s, master Top-K %d, "
                               "zeta_worker=%g, zeta_master=0, gradient pool of %d arrays; `value` is the one-stream "
                               "run (each step's kernels finish before the next step's start), the median of "
                               "`repeats` timed regions of `steps` steps each after `warmup` steps; the two-stream run "
                               "overlaps the worker compression of step t+1 with the server work of step t, which "
                               "supplied gradients allow and gradients computed at the new iterate would not"
                               % (n, d, [k for _, k in wk.worker_levels], wk.master_levels[0][1], wk.zeta_worker,
                                  npool),
                   "level_histogram_skip_then_levels": [int(v) for v in hist],
                   "repeats": args.repeats,
                   "ms_per_step_one_stream_with_kernel_events": t_ev[0] / args.steps * 1e3,
                   "candidates_kept_last_step_workers_master": cands,
                   "second_scans_workers_master": repairs[0]},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "zeta_sweep": sweep,
        "other_workloads": other,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
