"""CPU oracle for AdaCGD -- TEST INFRASTRUCTURE, not part of the product.

A plain, slow, step-by-step NumPy statement of what one iteration of DCGD with
master compression (Algorithm 1), written in three-point-compressor form
(Algorithm 2, "3PC-BD"), computes when the worker and master compressors are
AdaCGD compressors (Section 4.3, the AdaCGD definition) built from Top-K
sparsifiers (Section 2.1) and b-bit stochastic quantisers.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this module.  It shares no code with the HIP library and never calls it.

Arithmetic.  Every vector is stored in `dtype` (float32 = the precision the
device path stores in; float64 = "math mode" used to check the paper's
reductions exactly).  All reductions (squared norms, dot products, sums over
workers) are carried out in float64 or wider and rounded once to `dtype` where
a vector is stored.  Rounding points, in paper notation:
  v      = fl(x - h)                       argument of the compressor, Eq. (7)
  S      = sum_l (double v_l)^2            ||x - h||^2, first branch of the AdaCGD definition
  D      = sum_l (double fl(x_l - y_l))^2  ||x - y||^2, right side of Eq. (10)
  err_j  = sum_l (double v_l - double C_j(v)_l)^2   left side of Eq. (10)
  h_new  = fl(h + C_j(v))                  Eq. (7), literally "h + C(x - h)"
  g~     = fl(g~ + (sum_i C(v_i)) / n)     server aggregate, Algorithm 1 (incremental form)
  x      = fl(x - gamma * g)               Algorithm 1, iterate update
Parity status: every function below is pinned by tests/test_oracle_*.py
against closed forms, brute force, independent re-implementations of the
special cases the paper names (EF21, CLAG, LAG, plain GD) or published
known-answer values; full trajectories have no printed values in the paper and
are pinned only through those special cases and per-step invariants.
The b-bit quantiser is not defined by the paper: its definition here is a
reading (scaled stochastic uniform dithering with max-norm scale); it is
pinned against its own closed-form conditional expectation and the contractive
inequality of Definition 1, not against a paper value.  The block-wise variant
(one max-norm scale per block of B consecutive coordinates) is the same quantiser
applied to every block on its own; it is pinned against the plain one (block by
block, and B = d), the same closed form summed over the blocks, and Definition 1.
Rank-K (Section 2.1 names it beside Top-K for matrix-shaped arguments) is the
truncated singular value decomposition; how a gradient vector becomes a matrix is
a reading (row-major, c columns); it is pinned against the Eckart-Young optimum
(squared error = sum of the discarded squared singular values, not improved by any
other rank-K matrix tried), exact recovery of matrices of rank <= K, and the
contractive inequality with alpha = K / min(rows, columns).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

TOPK = 0
QUANT = 1
QUANT_BLOCK = 2      # level = (QUANT_BLOCK, (b, B)): b bits, one scale per block of B consecutive coordinates
RANK = 3             # level = (RANK, (K, c)): best rank-K approximation of the vector read as a (d/c) x c matrix

INIT_FULLGRAD = 0
INIT_ZERO = 1
INIT_COMPRESSED = 2


# --------------------------------------------------------------------------
# helpers
# --------------------------------------------------------------------------
def sum_squares(a) -> float:
    """sum_l (double a_l)^2, accumulated in extended precision (pairwise),
    rounded once to float64.  Each square of a float32 is exact in float64."""
    a = np.asarray(a, dtype=np.float64)
    sq = a * a
    return float(np.sum(sq.astype(np.longdouble)))


def sum_sq_diff(a, b) -> float:
    """sum_l (double a_l - double b_l)^2 in extended precision."""
    e = np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64)
    return float(np.sum((e * e).astype(np.longdouble)))


# --------------------------------------------------------------------------
# Top-K sparsifier (Section 2.1 names it; the tie order makes it a function)
# --------------------------------------------------------------------------
def magnitude_key(v: np.ndarray) -> np.ndarray:
    """Bit pattern of |v| as an unsigned integer.  For finite values this is
    monotone in |v|; +0 and -0 share key 0; no flush of denormals."""
    v = np.ascontiguousarray(v)
    if v.dtype == np.float32:
        return (v.view(np.uint32) & np.uint32(0x7FFFFFFF)).astype(np.int64)
    if v.dtype == np.float64:
        return (v.view(np.uint64) & np.uint64(0x7FFFFFFFFFFFFFFF)).astype(np.int64)
    raise TypeError(v.dtype)


def magnitude_order(v: np.ndarray) -> np.ndarray:
    """Indices of v in the total order (larger |v| first, then lower index):
    a full stable sort on the descending magnitude key."""
    return np.argsort(-magnitude_key(v), kind="stable")


def topk_support(v: np.ndarray, K: int, order: np.ndarray | None = None) -> np.ndarray:
    """Ascending indices of the K first elements in the total order."""
    if order is None:
        order = magnitude_order(v)
    return np.sort(order[:K])


def topk(v: np.ndarray, K: int, order: np.ndarray | None = None) -> np.ndarray:
    """Top-K(v): v on the support, 0 elsewhere."""
    c = np.zeros_like(v)
    idx = topk_support(v, K, order)
    c[idx] = v[idx]
    return c


# --------------------------------------------------------------------------
# Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw, SC'11)
# --------------------------------------------------------------------------
_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85
_MASK32 = np.uint64(0xFFFFFFFF)


def philox4x32_10(c0, c1, c2, c3, k0: int, k1: int):
    """Ten rounds of Philox-4x32 on arrays of counter words (uint32) with the
    scalar key (k0, k1).  Returns four uint32 arrays."""
    c0 = np.asarray(c0, dtype=np.uint64) & _MASK32
    c1 = np.asarray(c1, dtype=np.uint64) & _MASK32
    c2 = np.asarray(c2, dtype=np.uint64) & _MASK32
    c3 = np.asarray(c3, dtype=np.uint64) & _MASK32
    k0 &= 0xFFFFFFFF
    k1 &= 0xFFFFFFFF
    for r in range(10):
        if r > 0:
            k0 = (k0 + _PHILOX_W0) & 0xFFFFFFFF
            k1 = (k1 + _PHILOX_W1) & 0xFFFFFFFF
        p0 = _PHILOX_M0 * c0            # 64-bit products of 32-bit words
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK32
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0)
    return (c0.astype(np.uint32), c1.astype(np.uint32), c2.astype(np.uint32), c3.astype(np.uint32))


def dither_uniforms(d: int, seed: int, node: int, step: int) -> np.ndarray:
    """One uniform u_l in [0,1) per coordinate, a multiple of 2^-24.
    Counter = (l // 4, node, step, 0), key = the 64-bit seed; coordinate l takes
    output word l % 4.  `node` is the worker index, or 2^31 for the master."""
    q = (d + 3) // 4
    blk = np.arange(q, dtype=np.uint64)
    w = philox4x32_10(blk, np.full(q, node, dtype=np.uint64), np.full(q, step & 0xFFFFFFFF, dtype=np.uint64),
                      np.zeros(q, dtype=np.uint64), seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    words = np.stack(w, axis=1).reshape(-1)[:d]
    return (words >> np.uint32(8)).astype(np.float64) * 2.0 ** -24


# --------------------------------------------------------------------------
# b-bit stochastic quantiser (a reading; the paper only names "quantization")
# --------------------------------------------------------------------------
def quant_omega(d: int, b: int) -> float:
    s = 2 ** (b - 1) - 1
    return min(d / (4.0 * s * s), math.sqrt(d) / s)


def quant_alpha(d: int, b: int) -> float:
    """Contraction parameter of the scaled quantiser: alpha = 1 / (1 + omega)."""
    return 1.0 / (1.0 + quant_omega(d, b))


def quantize(v: np.ndarray, b: int, u: np.ndarray):
    """C_b(v) with s = 2^(b-1) - 1 magnitude levels and scale a = max |v|:
         r = (|v| / a) * s   (two roundings in v's dtype)
         xi = floor(r) + [u < r - floor(r)]
         C_b(v) = sign(v) * fl(xi * c),   c = fl(a / (s (1 + omega)))
    Returns (C_b(v), xi as int32 with the sign of v, c)."""
    dt = v.dtype.type
    d = v.shape[0]
    s = 2 ** (b - 1) - 1
    av = np.abs(v)
    a = av.max() if d else dt(0)
    if not (a > 0):
        return np.zeros_like(v), np.zeros(d, dtype=np.int32), dt(0)
    r = (av / a) * dt(s)
    fl = np.floor(r)
    p = r - fl
    xi = fl + (u.astype(v.dtype) < p)
    c = dt(float(a) / (s * (1.0 + quant_omega(d, b))))
    mag = (xi.astype(v.dtype) * c).astype(v.dtype)
    out = np.copysign(mag, v)
    codes = np.where(np.signbit(v), -xi, xi).astype(np.int32)
    return out, codes, c


def quant_expected_sqerr(v: np.ndarray, b: int) -> float:
    """E ||C_b(v) - v||^2 over the dither, in closed form (float64):
    with Delta = a/s, p_l the fractional part and w = omega,
      [sum_l Delta^2 p_l (1 - p_l)] / (1+w)^2 + (w/(1+w))^2 ||v||^2."""
    v = np.asarray(v, dtype=np.float64)
    d = v.shape[0]
    s = 2 ** (b - 1) - 1
    a = np.abs(v).max()
    if a == 0:
        return 0.0
    w = quant_omega(d, b)
    r = np.abs(v) / a * s
    p = r - np.floor(r)
    delta = a / s
    return float(np.sum(delta * delta * p * (1 - p)) / (1 + w) ** 2 + (w / (1 + w)) ** 2 * np.sum(v * v))


def quantize_block(v: np.ndarray, b: int, B: int, u: np.ndarray):
    """Block-wise C_b: the vector is cut into blocks of B consecutive coordinates (the last one may be
    shorter) and every block k is quantised on its own with the scale a_k = max |v| over the block:
         r = (|v| / a_k) * s,  xi = floor(r) + [u < r - floor(r)],  C(v) = sign(v) * fl(xi * c_k),
         c_k = fl(a_k / (s (1 + omega_B))),   omega_B = min(B / (4 s^2), sqrt(B) / s)
    i.e. the quantiser above with the block length in place of d (also for a shorter last block: omega
    grows with the length, so the nominal B keeps the block contractive).  A block of zeros gives zeros.
    Every block is then contractive in expectation with alpha_B = 1 / (1 + omega_B), and so is the whole.
    The dither u_l is the one of coordinate l (not restarted per block).
    Returns (C(v), signed codes xi as int32, scales c_k as an array of ceil(d / B) values)."""
    dt = v.dtype.type
    d = v.shape[0]
    s = 2 ** (b - 1) - 1
    nb = (d + B - 1) // B
    out = np.zeros_like(v)
    codes = np.zeros(d, dtype=np.int32)
    scales = np.zeros(nb, dtype=v.dtype)
    denom = s * (1.0 + quant_omega(B, b))
    for k in range(nb):
        lo, hi = k * B, min(d, (k + 1) * B)
        vb = v[lo:hi]
        av = np.abs(vb)
        a = av.max()
        if not (a > 0):
            continue
        r = (av / a) * dt(s)
        fl = np.floor(r)
        xi = fl + (u[lo:hi].astype(v.dtype) < (r - fl))
        c = dt(float(a) / denom)
        out[lo:hi] = np.copysign((xi.astype(v.dtype) * c).astype(v.dtype), vb)
        codes[lo:hi] = np.where(np.signbit(vb), -xi, xi).astype(np.int32)
        scales[k] = c
    return out, codes, scales


def quant_block_expected_sqerr(v: np.ndarray, b: int, B: int) -> float:
    """E ||C(v) - v||^2 of the block-wise quantiser over the dither: the closed form of the plain
    quantiser (with omega_B) summed over the blocks."""
    v = np.asarray(v, dtype=np.float64)
    d = v.shape[0]
    s = 2 ** (b - 1) - 1
    w = quant_omega(B, b)
    total = 0.0
    for lo in range(0, d, B):
        vb = v[lo:lo + B]
        a = np.abs(vb).max()
        if a == 0:
            continue
        r = np.abs(vb) / a * s
        p = r - np.floor(r)
        delta = a / s
        total += float(np.sum(delta * delta * p * (1 - p)) / (1 + w) ** 2 + (w / (1 + w)) ** 2 * np.sum(vb * vb))
    return total


# --------------------------------------------------------------------------
# Rank-K (Section 2.1): truncated singular value decomposition of the matrix-shaped argument
# --------------------------------------------------------------------------
def rank_k(v: np.ndarray, K: int, c: int):
    """Best rank-K approximation (in the Frobenius norm) of v read row-major as a matrix X of
    d/c rows and c columns: X_K = sum_{k<K} sigma_k u_k v_k^T from a singular value decomposition in
    float64, rounded once to v's dtype.  It is unique when sigma_K > sigma_{K+1}.
    Returns (C(v) as a vector of length d, the singular values)."""
    d = v.shape[0]
    assert d % c == 0 and 1 <= K <= c
    X = np.asarray(v, dtype=np.float64).reshape(d // c, c)
    U, sig, Vt = np.linalg.svd(X, full_matrices=False)
    XK = (U[:, :K] * sig[:K]) @ Vt[:K]
    return XK.reshape(d).astype(v.dtype), sig


# --------------------------------------------------------------------------
# level sets
# --------------------------------------------------------------------------
def level_alpha(level, d: int) -> float:
    kind, param = level
    if kind == TOPK:
        return param / d
    if kind == QUANT:
        return quant_alpha(d, param)
    if kind == RANK:
        K, c = param
        return K / min(c, d // c)     # ||X_K - X||_F^2 = sum of the min(r, c) - K smallest sigma^2 <= (1 - K/min(r, c)) ||X||_F^2
    b, B = param
    return quant_alpha(B, b)          # every block is contractive with the parameter of a length-B vector


def check_levels(levels, d: int):
    """The AdaCGD definition orders levels by alpha_1 <= ... <= alpha_m."""
    al = [level_alpha(lv, d) for lv in levels]
    return all(al[i] <= al[i + 1] for i in range(len(al) - 1))


# --------------------------------------------------------------------------
# the AdaCGD compressor C^AC_{h,y}(x)  (Section 4.3)
# --------------------------------------------------------------------------
@dataclass
class CompressResult:
    level: int                 # 0 = skip (returns h), 1..m = level applied
    S: float                   # ||x - h||^2
    D: float                   # ||x - y||^2
    err: list                  # err_j = ||x - C^{EF,j}_{h,y}(x)||^2 for j = 1..m
    h_new: np.ndarray          # C^AC_{h,y}(x)
    msg_idx: np.ndarray        # ascending coordinates sent (Top-K level), else empty
    msg_val: np.ndarray        # values sent (Top-K level)
    dense: np.ndarray | None   # C_b(v) when a quantiser level is applied
    codes: np.ndarray | None = None
    scale: float = 0.0
    scales: np.ndarray | None = None   # block-wise quantiser level: one scale per block
    sigma: np.ndarray | None = None    # Rank-K level: the singular values of the matrix-shaped argument
    margins: list = field(default_factory=list)   # |lhs - tau| / max(tau, tiny) of every comparison made


def adacgd_compress(h, y, x, levels, zeta, *, seed=0, node=0, step=0, D_given=None, v_given=None,
                    triggers=None) -> CompressResult:
    """Apply the AdaCGD compressor to x with stored estimator h and previous
    point y.  `levels` is the ordered list [(kind, param), ...].
    v_given / D_given replace x - h and ||x - y||^2 when the caller supplies
    the difference vector directly.

    `triggers` generalises the conditions of the cascade the way the Ada3PC
    definition (Section 4.2) and Lemma 2 allow: any conditions P_0..P_{m-1} may
    guard the levels.  The family here is
        P_j :  err_j <= zeta_j ||x - y||^2 + eta_j ||x - h||^2,   err_0 = ||x - h||^2,
    given as m pairs (zeta_j, eta_j), j = 0 (keep h) .. m-1; the last level is
    unconditional.  None means (zeta, 0) for every j: the AdaCGD definition."""
    dt = h.dtype
    d = h.shape[0]
    v = np.asarray(v_given, dtype=dt) if v_given is not None else (x - h).astype(dt)
    S = sum_squares(v)
    same_terms = False        # x - h and x - y are the same vector: S and D are the same sum
    if D_given is not None:
        D = float(D_given)
    else:
        w = (x - y).astype(dt)
        D = sum_squares(w)
        same_terms = bool(np.array_equal(v, w))
    m = len(levels)
    if triggers is None:
        triggers = [(zeta, 0.0)] * m
    assert len(triggers) == m
    # the constants are held in the storage dtype; each product and the sum is rounded once (float64)
    taus = [float(np.float64(dt.type(z))) * D + float(np.float64(dt.type(e))) * S for z, e in triggers]

    order = None
    u = None
    cands = []
    err = []
    for kind, param in levels:
        if kind == TOPK:
            if order is None:
                order = magnitude_order(v)
            c = topk(v, param, order)
            cands.append(("topk", c, topk_support(v, param, order)))
        elif kind == RANK:
            c, sig = rank_k(v, param[0], param[1])
            cands.append(("rank", c, None, sig))
        else:
            if u is None:
                u = dither_uniforms(d, seed, node, step)
            if kind == QUANT:
                c, codes, scale = quantize(v, param, u)
            else:
                c, codes, scale = quantize_block(v, param[0], param[1], u)      # scale: one per block
            cands.append(("quant", c, codes, scale))
        err.append(sum_sq_diff(v, c))

    margins = []

    def holds(lhs, tau):
        # relative distance from equality; 0 == 0 is exact on any summation order (every term is zero)
        margins.append(float("inf") if lhs == 0.0 and tau == 0.0 else abs(lhs - tau) / max(tau, 1e-300))
        return lhs <= tau

    if same_terms and taus[0] == D and float(dt.type(triggers[0][1])) == 0.0:
        margins.append(float("inf"))      # S == D term by term: the comparison is S <= S
        first = True
    else:
        first = holds(S, taus[0])
    if first:
        level = 0
    else:
        level = m
        for j in range(1, m):
            if holds(err[j - 1], taus[j]):
                level = j
                break

    empty_i = np.zeros(0, dtype=np.int32)
    empty_v = np.zeros(0, dtype=dt)
    if level == 0:
        return CompressResult(0, S, D, err, h.copy(), empty_i, empty_v, None, margins=margins)
    cand = cands[level - 1]
    if cand[0] == "topk":
        idx = cand[2]
        h_new = h.copy()
        h_new[idx] = (h[idx] + v[idx]).astype(dt)
        return CompressResult(level, S, D, err, h_new, idx.astype(np.int32), v[idx].copy(), None, margins=margins)
    c = cand[1]
    h_new = (h + c).astype(dt)
    if cand[0] == "rank":
        return CompressResult(level, S, D, err, h_new, empty_i, empty_v, c, sigma=cand[3], margins=margins)
    blockwise = np.ndim(cand[3]) > 0
    return CompressResult(level, S, D, err, h_new, empty_i, empty_v, c, codes=cand[2],
                          scale=0.0 if blockwise else float(cand[3]), scales=cand[3] if blockwise else None,
                          margins=margins)


# --------------------------------------------------------------------------
# objective of the experiments (Section 6): logistic loss + nonconvex regulariser
# --------------------------------------------------------------------------
def logistic_loss(A, labels, x, lam) -> float:
    """f_i(x) = (1/N_i) sum_l log(1 + exp(-y_l a_l^T x)) + lam sum_j x_j^2 / (1 + x_j^2)."""
    A = np.asarray(A, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    yl = np.asarray(labels, dtype=np.float64)
    z = A @ x
    return float(np.mean(np.logaddexp(0.0, -yl * z)) + lam * np.sum(x * x / (1.0 + x * x)))


def logistic_grad(A, labels, x, lam, dtype=np.float32) -> np.ndarray:
    """grad f_i(x) = -(1/N_i) sum_l y_l a_l / (1 + exp(y_l a_l^T x)) + 2 lam x_j / (1 + x_j^2)^2,
    all in float64, rounded once to `dtype`."""
    A64 = np.asarray(A, dtype=np.float64)
    x64 = np.asarray(x, dtype=np.float64)
    yl = np.asarray(labels, dtype=np.float64)
    z = A64 @ x64
    with np.errstate(over="ignore"):
        s = -yl / (1.0 + np.exp(yl * z)) / A64.shape[0]
    g = A64.T @ s + 2.0 * lam * x64 / (1.0 + x64 * x64) ** 2
    return g.astype(dtype)


# --------------------------------------------------------------------------
# Algorithm 1 / Algorithm 2 driver
# --------------------------------------------------------------------------
class AdaCGDOracle:
    """State and one-iteration update of DCGD with master compression where
    both compressors are AdaCGD compressors (Algorithm 2 gives the h and y of
    each: worker i uses h = g~_i^t, y = grad f_i(x^t); the master uses
    h = g^t, y = g~^t)."""

    def __init__(self, *, n, d, gamma, worker_levels, zeta_worker, master_levels=(), zeta_master=0.0,
                 seed=0, dtype=np.float32, shards=None, lam=0.1, worker_triggers=None, master_triggers=None):
        self.n, self.d = int(n), int(d)
        self.dt = np.dtype(dtype)
        self.gamma = float(np.float64(self.dt.type(gamma)))
        self.wl = [tuple(l) for l in worker_levels]
        self.ml = [tuple(l) for l in master_levels]
        self.zw, self.zm = zeta_worker, zeta_master
        self.tw, self.tm = worker_triggers, master_triggers
        self.seed = int(seed)
        self.shards = shards            # list of (A_i, labels_i) or None
        self.lam = float(np.float64(self.dt.type(lam)))
        self.t = 0
        # how the independent per-worker compressions of a step are evaluated: the built-in map, or for
        # instance a thread pool's map at large sizes (the results do not depend on it)
        self.worker_map = map
        self.level_hist_w = np.zeros(len(self.wl) + 1, dtype=np.int64)
        self.level_hist_m = np.zeros(len(self.ml) + 1, dtype=np.int64)
        self.last = None

    # -- gradients ---------------------------------------------------------
    def local_grads(self, x):
        return np.stack(list(self.worker_map(lambda sh: logistic_grad(sh[0], sh[1], x, self.lam, self.dt), self.shards)))

    # -- input line of Algorithm 1 ----------------------------------------
    def init(self, x0, grads0=None, init_mode=INIT_FULLGRAD):
        dt = self.dt
        self.x = np.asarray(x0, dtype=dt).copy()
        if grads0 is None and self.shards is not None:
            grads0 = self.local_grads(self.x)
        if grads0 is not None:
            self.y = np.asarray(grads0, dtype=dt).copy()       # grad f_i(x^0)
        else:
            self.y = np.zeros((self.n, self.d), dtype=dt)
        if init_mode == INIT_FULLGRAD:
            self.gi = self.y.copy()
        elif init_mode == INIT_ZERO:
            self.gi = np.zeros((self.n, self.d), dtype=dt)
        elif init_mode == INIT_COMPRESSED:
            # g~_i^0 = C_m(grad f_i(x^0)), C_m the last level: the start of CLAG and EF21 (Section 2.3)
            kind, param = self.wl[-1]
            assert kind == TOPK
            self.gi = np.stack([topk(self.y[i], param) for i in range(self.n)])
        else:
            raise ValueError(init_mode)
        acc = np.zeros(self.d, dtype=np.float64)
        for i in range(self.n):
            acc += self.gi[i].astype(np.float64)
        self.gt = (acc / self.n).astype(dt)       # g~^0 = (1/n) sum g~_i^0
        self.gt_prev = self.gt.copy()
        self.g = self.gt.copy()                   # g^0
        self.t = 0

    # -- one iteration t -> t+1 -------------------------------------------
    def step(self, grads=None, diffs=None, D=None):
        dt = self.dt
        n, d = self.n, self.d
        # x^{t+1} = x^t - gamma g^t
        self.x = (self.x.astype(np.float64) - self.gamma * self.g.astype(np.float64)).astype(dt)
        # grad f_i(x^{t+1})
        if diffs is None:
            if grads is None:
                grads = self.local_grads(self.x)
            grads = np.asarray(grads, dtype=dt)
        # "for all devices in parallel" (Algorithm 1): the n compressions are independent of each other
        def one(i):
            if diffs is not None:
                return adacgd_compress(self.gi[i], None, None, self.wl, self.zw, seed=self.seed, node=i, step=self.t,
                                       D_given=D[i], v_given=diffs[i], triggers=self.tw)
            return adacgd_compress(self.gi[i], self.y[i], grads[i], self.wl, self.zw, seed=self.seed, node=i,
                                   step=self.t, triggers=self.tw)
        res = list(self.worker_map(one, range(n)))
        acc = np.zeros(d, dtype=np.float64)
        for i in range(n):                        # messages are added in ascending worker index
            r = res[i]
            self.gi[i] = r.h_new
            if r.level > 0:
                if r.dense is not None:
                    acc += r.dense.astype(np.float64)
                else:
                    acc[r.msg_idx] += r.msg_val.astype(np.float64)
            self.level_hist_w[r.level] += 1
        if diffs is None:
            self.y = grads.copy()                 # y_i <- grad f_i(x^{t+1}), on skip too
        # server: g~^{t+1} = g~^t + (1/n) sum_i messages  (== (1/n) sum_i g~_i^{t+1})
        gt_new = (self.gt.astype(np.float64) + acc / n).astype(dt)
        self.gt_prev = self.gt
        self.gt = gt_new
        # master: g^{t+1} = C^M_{g^t, g~^t}(g~^{t+1})
        if len(self.ml) == 0:
            self.g = self.gt.copy()
            rm = None
        else:
            rm = adacgd_compress(self.g, self.gt_prev, self.gt, self.ml, self.zm, seed=self.seed, node=1 << 31,
                                 step=self.t, triggers=self.tm)
            self.g = rm.h_new
            self.level_hist_m[rm.level] += 1
        self.t += 1
        self.last = (res, rm)
        return res, rm

    # -- communication counters -------------------------------------------
    @staticmethod
    def message_bits(level, levels, d):
        """Bits of one message: level id + payload.  Top-K: K (value, index)
        pairs; b-bit: d codes plus one float scale (block-wise: one per block); skip: the id only."""
        m = len(levels)
        idb = max(1, math.ceil(math.log2(m + 1)))
        if level == 0:
            return idb
        kind, param = levels[level - 1]
        if kind == TOPK:
            return idb + param * (32 + max(1, math.ceil(math.log2(d))))
        if kind == QUANT:
            return idb + d * param + 32
        if kind == RANK:
            K, c = param
            return idb + 32 * K * (d // c + c)            # K left factors (scaled) of d/c floats, K right factors of c
        b, B = param
        return idb + d * b + 32 * ((d + B - 1) // B)      # one float scale per block

    @staticmethod
    def message_values(level, levels, d):
        if level == 0:
            return 0
        kind, param = levels[level - 1]
        if kind == RANK:
            return param[0] * (d // param[1] + param[1])
        return param if kind == TOPK else d
