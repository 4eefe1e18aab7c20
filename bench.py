#!/usr/bin/env python3
"""Benchmark of the AdaCGD hot path on one MI355X.

A step is one full iteration of Algorithm 2 on the model-sized workload (n = 16
workers, d = 11.2 M, Top-K levels at {1e-4, 1e-3, 1e-2, 5e-2} d, master Top-K at
1e-2 d): iterate update, worker compression with level choice for all workers,
server aggregation, master compression.  The per-worker gradients are supplied
(seeded synthetic vectors already resident in HBM), as that workload defines them.

Prints one JSON line: throughput (compressed floats per second = n d steps / s),
the roofline position of the worker compression kernels from HIP-event timings
taken inside the library, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per step of the worker-side selection kernels on the default workload, from the
# rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised in profiles/model_sized_n16_d11200000_hbm_traffic.md
# (reads scaled by 2.0, writes by 1.0, as calibrated there).  Valid only for the default
# arguments and for the kernels as they were when the counters were taken.
MEASURED_TRAFFIC_BYTES = 3086.4e6
MEASURED_TRAFFIC_KERNELS = "w_sample+w_scan+w_filter+w_gather+w_select+w_tally+w_compact"


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


def extra_kernel_stress(E, W, torch, steps=50, warmup=4):
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
    return {"workload": "kernel stress: n=%d, d=%d, difference vectors exp(N(0,1)) * t3, levels %s, master Top-%d"
                        % (wk.n, wk.d, wk.worker_levels, wk.master_levels[0][1]),
            "steps": steps, "ms_per_step": dt / steps * 1e3, "floats_per_sec": wk.n * wk.d * steps / dt,
            "level_histogram_skip_then_levels": [int(v) for v in hist], "kernels_avg_ms": kms,
            "note": "one stream, HIP events around every kernel"}


def extra_federated(E, W, torch, n, steps=10, warmup=2):
    """Secondary workload: logistic-regression shards (engine computes the gradients), d=65536, 32 samples each."""
    wl = W.federated(n=n)
    A, labels = torch.from_numpy(wl.A).cuda(), torch.from_numpy(wl.labels).cuda()
    x0 = torch.zeros(wl.d, dtype=torch.float32, device="cuda")
    eng = E.AdaCGD(n=wl.n, d=wl.d, gamma=wl.gamma, lam=wl.lam, worker_levels=wl.worker_levels,
                   zeta_worker=wl.zeta_worker, master_levels=wl.master_levels, zeta_master=wl.zeta_master,
                   grad_mode=E.GRAD_LOGISTIC, A=A, labels=labels, shard_offsets=wl.shard_offsets, x0=x0, seed=5,
                   flags=E.FLAG_KERNEL_TIMING)
    dt, hist, kms = _timed_steps(eng, E, torch, lambda t: eng.step(), warmup, steps)
    eng.close()
    a_bytes = float(wl.A.nbytes)
    grad_ms = kms.get("grad_margin", 0.0) + kms.get("grad_cols", 0.0)
    return {"workload": "federated logistic regression: n=%d workers, d=%d, %d samples each, "
                        "levels %s, master Top-%d" % (wl.n, wl.d, wl.A.shape[0] // wl.n, wl.worker_levels,
                                                      wl.master_levels[0][1]),
            "steps": steps, "ms_per_step": dt / steps * 1e3, "floats_per_sec": wl.n * wl.d * steps / dt,
            "level_histogram_skip_then_levels": [int(v) for v in hist], "kernels_avg_ms": kms,
            "gradient_kernels": {"algorithmic_bytes": 2 * a_bytes, "avg_ms": grad_ms,
                                 "GB/s": 2 * a_bytes / (grad_ms * 1e-3) / 1e9 if grad_ms else None,
                                 "frac_of_8TBps": 2 * a_bytes / (grad_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if grad_ms else None},
            "note": "one stream, HIP events around every kernel"}


def extra_sparse_features(E, W, torch, steps=20, warmup=3):
    """Secondary workload: logistic regression on binary features kept as compressed sparse rows."""
    wl = W.sparse_features()
    nnz = int(wl.csr[0][-1])
    rows = wl.labels.shape[0]
    x0 = torch.zeros(wl.d, dtype=torch.float32, device="cuda")
    eng = E.AdaCGD(n=wl.n, d=wl.d, gamma=wl.gamma, lam=wl.lam, worker_levels=wl.worker_levels,
                   zeta_worker=wl.zeta_worker, master_levels=wl.master_levels, zeta_master=wl.zeta_master,
                   grad_mode=E.GRAD_LOGISTIC_CSR, labels=torch.from_numpy(wl.labels).cuda(),
                   shard_offsets=wl.shard_offsets, csr=wl.csr, x0=x0, flags=E.FLAG_KERNEL_TIMING)
    dt, hist, kms = _timed_steps(eng, E, torch, lambda t: eng.step(), warmup, steps)
    eng.close()
    # stored entries: column + gathered x (margins), row + gathered fp64 margin (column sums); per row the
    # pointer, label and margin; per (worker, column) the column pointer and the gradient written
    alg = nnz * (4 + 4 + 4 + 8) + rows * (8 + 4 + 8) + wl.n * wl.d * (4 + 4)
    grad_ms = kms.get("grad_margin", 0.0) + kms.get("grad_cols", 0.0)
    return {"workload": "sparse binary features: n=%d workers, d=%d, %d rows each, %d stored entries per row, "
                        "Top-K levels %s, master Top-%d" % (wl.n, wl.d, rows // wl.n, nnz // rows,
                                                            [k for _, k in wl.worker_levels], wl.master_levels[0][1]),
            "steps": steps, "ms_per_step": dt / steps * 1e3, "floats_per_sec": wl.n * wl.d * steps / dt,
            "level_histogram_skip_then_levels": [int(v) for v in hist], "kernels_avg_ms": kms,
            "gradient_kernels": {"algorithmic_bytes": alg, "avg_ms": grad_ms,
                                 "GB/s": alg / (grad_ms * 1e-3) / 1e9 if grad_ms else None,
                                 "dense_matrix_bytes_for_comparison": 4.0 * rows * wl.d},
            "note": "one stream, HIP events around every kernel"}


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
            "kernel_launches_per_step": launches,
            "level_histogram_skip_then_levels_since_init": [int(v) for v in hist],
            "note": "a step is four short dependent kernels: latency-bound, no roofline applies"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--pool", type=int, default=4, help="distinct gradient arrays cycled through")
    ap.add_argument("--zeta", type=float, default=1.0)
    ap.add_argument("--n", type=int, default=16)
    ap.add_argument("--d", type=int, default=11_200_000)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the secondary workloads")
    ap.add_argument("--federated-n", type=int, default=1000,
                    help="workers of the secondary federated workload (1000 = the full configuration, 8.4 GB of features)")
    ap.add_argument("--secondary", choices=["kernel_stress", "federated", "sparse_features"],
                    help="run only this secondary workload and print its record (for profiling it on its own)")
    ap.add_argument("--no-overlap", action="store_true",
                    help="run the worker and server chains on one stream (the kernel-timing pass always does)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (all n workers are batched on it); "
              "--gpus > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2211_00188_amd import engine as E
    from paper_2211_00188_amd import workloads as W

    torch.cuda.set_device(0)
    if args.secondary:
        rec = {"kernel_stress": lambda: extra_kernel_stress(E, W, torch),
               "federated": lambda: extra_federated(E, W, torch, args.federated_n),
               "sparse_features": lambda: extra_sparse_features(E, W, torch)}[args.secondary]()
        print(json.dumps({"secondary_workload": rec}))
        return
    wk = W.model_sized(n=args.n, d=args.d, zeta=args.zeta)
    n, d = wk.n, wk.d
    gen = W.ModelSizedGrads(wk)
    host0 = gen.next().copy()
    g0 = torch.from_numpy(host0).cuda()
    pool_host = []
    pool = []
    for _ in range(args.pool):
        a = gen.next().copy()
        if len(pool_host) < 2:
            pool_host.append(a)
        pool.append(torch.from_numpy(a).cuda())
    x0 = torch.zeros(d, dtype=torch.float32, device="cuda")

    repairs = []

    def run(flags, steps, warmup):
        eng = E.AdaCGD(n=n, d=d, gamma=0.1, worker_levels=wk.worker_levels, zeta_worker=wk.zeta_worker,
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
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            eng.step(pool[t % len(pool)])
            t += 1
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        hist = eng.state(E.F_LEVEL_HIST).astype(np.int64) - h0
        kms = eng.kernel_ms() if flags & E.FLAG_KERNEL_TIMING else None
        repairs.append([int(v) for v in eng.state(E.F_REPAIRS)])
        eng.close()
        del eng
        torch.cuda.empty_cache()
        return dt, hist, kms

    dt, hist, _ = run(0 if args.no_overlap else E.FLAG_OVERLAP, args.steps, args.warmup)
    dt_ev, hist_ev, kms = run(E.FLAG_KERNEL_TIMING, args.steps, args.warmup)

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
    group_ms = sum(per_kernel[k]["avg_ms"] for k in group if k in per_kernel)
    achieved = alg_bytes_step / (group_ms * 1e-3) / 1e9
    group = [k for k in group if k in per_kernel]
    dom = max(group, key=lambda k: per_kernel[k]["avg_ms"])
    dom_bytes = {"w_scan": 12.0 * n * d, "w_filter": 8.0 * n * d}.get(dom, 0.0)
    default_workload = (args.n, args.d, args.zeta, args.pool) == (16, 11_200_000, 1.0, 4)
    traffic = MEASURED_TRAFFIC_BYTES if default_workload and "+".join(group) == MEASURED_TRAFFIC_KERNELS else None
    roofline = {
        "bound": "hbm", "kernel": "+".join(group), "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
        "traffic_GBps": traffic / (group_ms * 1e-3) / 1e9 if traffic else None,
        "algorithmic_bytes_per_step": alg_bytes_step, "avg_ms_per_step": group_ms,
        "dominant_kernel": {"name": dom, "avg_ms": per_kernel[dom]["avg_ms"],
                            "bytes_read_per_launch": dom_bytes,
                            "GB/s": dom_bytes / (per_kernel[dom]["avg_ms"] * 1e-3) / 1e9,
                            "frac": dom_bytes / (per_kernel[dom]["avg_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "kernels_avg_ms": {k: round(v["avg_ms"], 5) for k, v in per_kernel.items()},
    }

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import adacgd_oracle as O
        sample = list(range(max(1, min(8, n))))        # about 10 s of single-core NumPy work at d = 11.2 M
        t0 = time.perf_counter()
        for i in sample:
            O.adacgd_compress(host0[i], host0[i], pool_host[0][i], wk.worker_levels, wk.zeta_worker)
        ct = time.perf_counter() - t0
        cpu = {"value": len(sample) * d / ct, "unit": "floats/s", "cores": 1, "kind": "oracle",
               "sample": "worker compression step (all levels, level choice, estimator update) of %d of the %d "
                         "workers at d=%d, one step; the server and master steps are not included"
                         % (len(sample), n, d),
               "seconds": ct}

    npool = len(pool)
    del pool, g0, x0
    torch.cuda.empty_cache()
    other = []
    if not args.no_extras:
        other.append(extra_kernel_stress(E, W, torch))
        other.append(extra_federated(E, W, torch, args.federated_n))
        other.append(extra_small_logistic(E, W, torch, W.tiny(), 2000))
        other.append(extra_small_logistic(E, W, torch, W.sparse_logreg(), 2000))
        other.append(extra_small_logistic(E, W, torch, W.sparse_logreg(), 2000, sparse_rows=True))
        other.append(extra_sparse_features(E, W, torch))

    out = {
        "metric": "adacgd_compressed_floats_per_sec", "value": floats_per_s, "unit": "floats/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "steps_per_sec": steps_per_s,
        "config": {"workload": "model-sized vectors: n=%d workers, d=%d, external gradients "
                               "(shared AR(1) drift + 0.5 * per-worker offset), Top-K levels %s, master Top-K %d, "
                               "zeta_worker=%g, zeta_master=0, gradient pool of %d arrays"
                               % (n, d, [k for _, k in wk.worker_levels], wk.master_levels[0][1], wk.zeta_worker,
                                  npool),
                   "level_histogram_skip_then_levels": [int(v) for v in hist],
                   "streams": "one" if args.no_overlap else
                   "two (worker compression of step t+1 overlaps aggregation + master compression of step t)",
                   "ms_per_step_one_stream_with_kernel_events": dt_ev / args.steps * 1e3,
                   "second_scans_workers_master": repairs[0]},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "other_workloads": other,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
