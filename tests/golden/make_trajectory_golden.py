"""Writes tests/golden/trajectory_tiny_external.txt: the level choices, message supports and a checksum
of every state vector of a short AdaCGD run, computed by the CPU oracle alone on inputs from the seeded
generators.  The file guards the oracle against accidental drift (a CPU test recomputes it) and gives the
GPU path a stored reference.  Run from the repository root:  python tests/golden/make_trajectory_golden.py"""
import hashlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import adacgd_oracle as O  # noqa: E402

N, D, STEPS = 3, 50, 6
WORKER_LEVELS = [(O.TOPK, 1), (O.TOPK, 5), (O.QUANT, 4), (O.TOPK, 25)]
MASTER_LEVELS = [(O.TOPK, 10)]
ZETA_W, ZETA_M, GAMMA, SEED = 1.0, 0.5, 0.05, 7


def inputs():
    rng = np.random.Generator(np.random.Philox(20221101))
    grads = [rng.standard_normal((N, D), dtype=np.float32)]
    for t in range(STEPS):
        scale = np.float32(10.0 ** rng.uniform(-1.5, 0))
        grads.append((grads[-1] + scale * rng.standard_normal((N, D), dtype=np.float32)).astype(np.float32))
    x0 = rng.standard_normal(D, dtype=np.float32)
    return x0, grads


def digest(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()[:16]


def lines():
    x0, grads = inputs()
    orc = O.AdaCGDOracle(n=N, d=D, gamma=GAMMA, worker_levels=WORKER_LEVELS, zeta_worker=ZETA_W,
                         master_levels=MASTER_LEVELS, zeta_master=ZETA_M, seed=SEED)
    orc.init(x0, grads[0], O.INIT_FULLGRAD)
    out = ["# step | worker levels | master level | per worker: message coordinates | sha256/16 of x, g, g~, g~_i (fp32 bytes)"]
    for t in range(1, STEPS + 1):
        res, rm = orc.step(grads=grads[t])
        msgs = ";".join(",".join(str(int(i)) for i in r.msg_idx) for r in res)
        out.append("%d | %s | %d | %s | %s %s %s %s" % (t, " ".join(str(r.level) for r in res), rm.level, msgs,
                                                      digest(orc.x), digest(orc.g), digest(orc.gt), digest(orc.gi)))
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "trajectory_tiny_external.txt")
    with open(path, "w") as f:
        f.write("\n".join(lines()) + "\n")
    print("wrote", path)
