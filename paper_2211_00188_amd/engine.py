"""ctypes binding of libadacgd.so -- argument marshalling only.

Same entry points as include/adacgd.h (adacgd_workspace_bytes / adacgd_init /
adacgd_step / adacgd_state / adacgd_destroy).  PyTorch supplies device memory
(one uint8 workspace tensor per context) and the stream; every step of the
method runs in the library's HIP kernels.  There is no CPU fallback: if the
library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libadacgd.so")

TOPK, QUANT, QUANT_BLOCK, RANK = 0, 1, 2, 3      # levels: (QUANT_BLOCK, (b, B)), (RANK, (K, c))
GRAD_LOGISTIC, GRAD_EXTERNAL, DIFF_EXTERNAL, GRAD_LOGISTIC_CSR = 0, 1, 2, 3
INIT_FULLGRAD, INIT_ZERO, INIT_COMPRESSED = 0, 1, 2
FLAG_ANY_LEVEL_ORDER, FLAG_RETAIN_EXT, FLAG_KERNEL_TIMING, FLAG_TWO_PASS, FLAG_OVERLAP = 1, 2, 4, 8, 16
MAX_LEVELS = 16

(F_X, F_G, F_GTILDE, F_GTILDE_PREV, F_GI, F_PREV_GRAD, F_LEVEL, F_SQNORM, F_D, F_ERR, F_MSG_COUNT, F_MSG_IDX,
 F_MSG_VAL, F_M_LEVEL, F_M_SQNORM, F_M_D, F_M_ERR, F_M_MSG_COUNT, F_M_MSG_IDX, F_M_MSG_VAL, F_STEP, F_LEVEL_HIST,
 F_M_LEVEL_HIST, F_COMM, F_QCODES, F_QSCALE, F_KERNEL_MS, F_GRAD, F_REPAIRS, F_ESTIMATOR_ERR,
 F_CANDIDATES, F_QBSCALE, F_RANK_SPECTRUM) = range(33)

KERNELS = ["xupdate", "grad_margin", "grad_cols", "aggregate",
           "w_sample", "w_scan", "w_filter", "w_gather", "w_select", "w_tally", "w_compact", "w_qapply",
           "m_sample", "m_scan", "m_filter", "m_gather", "m_select", "m_tally", "m_compact", "m_qapply",
           "w_rank", "m_rank", "w_eig", "m_eig"]

EXPORTS = ["adacgd_workspace_bytes", "adacgd_init", "adacgd_init_static", "adacgd_step", "adacgd_state", "adacgd_set_state",
           "adacgd_destroy", "adacgd_last_error"]


class Level(C.Structure):
    _fields_ = [("kind", C.c_int32), ("block", C.c_int32), ("param", C.c_int64)]


class Trigger(C.Structure):
    _fields_ = [("zeta", C.c_float), ("eta", C.c_float)]


class Config(C.Structure):
    _fields_ = [
        ("n", C.c_int64), ("d", C.c_int64), ("grad_mode", C.c_int32), ("init_mode", C.c_int32),
        ("A", C.c_void_p), ("labels", C.c_void_p), ("shard_offsets", C.c_void_p), ("x0", C.c_void_p),
        ("grad0", C.c_void_p), ("lam", C.c_float), ("gamma", C.c_float),
        ("worker_levels", C.POINTER(Level)), ("m_worker", C.c_int32), ("zeta_worker", C.c_float),
        ("master_levels", C.POINTER(Level)), ("m_master", C.c_int32), ("zeta_master", C.c_float),
        ("seed", C.c_uint64), ("flags", C.c_uint32), ("pad", C.c_uint32),
        ("stream", C.c_void_p), ("workspace", C.c_void_p), ("workspace_bytes", C.c_int64),
        ("worker_triggers", C.POINTER(Trigger)), ("master_triggers", C.POINTER(Trigger)),
        ("csr_row_ptr", C.c_void_p), ("csr_col", C.c_void_p), ("csr_val", C.c_void_p),
    ]


class AdaCGDError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("adacgd error %d: %s" % (code, msg))
        self.code = code


_lib = None


def load_library():
    """Loads the native library; raises if it is missing (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                LIB_PATH + " is not built; run `python -m paper_2211_00188_amd.build` (needs hipcc)")
        # PyTorch bundles its own HIP runtime and owns the device memory this library works
        # on: import it first so that both share that one runtime (two runtimes in a
        # process do not both see the GPU).
        import torch  # noqa: F401
        lib = C.CDLL(LIB_PATH)
        lib.adacgd_workspace_bytes.argtypes = [C.POINTER(Config), C.POINTER(C.c_int64)]
        lib.adacgd_workspace_bytes.restype = C.c_int
        lib.adacgd_init.argtypes = [C.POINTER(Config), C.POINTER(C.c_void_p)]
        lib.adacgd_init.restype = C.c_int
        lib.adacgd_init_static.argtypes = [C.POINTER(Config), C.POINTER(C.c_void_p)]
        lib.adacgd_init_static.restype = C.c_int
        lib.adacgd_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]
        lib.adacgd_step.restype = C.c_int
        lib.adacgd_state.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int64, C.c_int32]
        lib.adacgd_state.restype = C.c_int
        lib.adacgd_set_state.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int64, C.c_int32]
        lib.adacgd_set_state.restype = C.c_int
        lib.adacgd_destroy.argtypes = [C.c_void_p]
        lib.adacgd_destroy.restype = C.c_int
        lib.adacgd_last_error.argtypes = [C.c_void_p]
        lib.adacgd_last_error.restype = C.c_char_p
        _lib = lib
    return _lib


def _levels(levels):
    arr = (Level * max(1, len(levels)))()
    for j, (kind, param) in enumerate(levels):
        block = 0
        if int(kind) in (QUANT_BLOCK, RANK):
            param, block = param                   # (bits, block length) / (rank, columns)
        arr[j].kind, arr[j].block, arr[j].param = int(kind), int(block), int(param)
    return arr


def _triggers(trig, m):
    if trig is None:
        return None
    trig = list(trig)
    if len(trig) != m:
        raise ValueError("need one (zeta, eta) pair per cascade position 0..m-1: %d given for %d levels" % (len(trig), m))
    arr = (Trigger * max(1, m))()
    for j, (z, e) in enumerate(trig):
        arr[j].zeta, arr[j].eta = float(z), float(e)
    return arr


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def make_config(*, n, d, worker_levels, zeta_worker, master_levels=(), zeta_master=0.0, gamma=0.1, lam=0.1,
                grad_mode=GRAD_EXTERNAL, init_mode=INIT_FULLGRAD, A=None, labels=None, shard_offsets=None,
                x0=None, grad0=None, seed=0, flags=0, stream=0, worker_triggers=None, master_triggers=None,
                csr=None):
    """Fills an adacgd_config.  Tensor arguments are CUDA float32 tensors (borrowed);
    shard_offsets is a host int64 NumPy array; csr = (row_ptr, col, val or None) are host
    NumPy arrays (GRAD_LOGISTIC_CSR).  Returns (cfg, keepalive)."""
    cfg = Config()
    wl, ml = _levels(list(worker_levels)), _levels(list(master_levels))
    so = None if shard_offsets is None else np.ascontiguousarray(shard_offsets, dtype=np.int64)
    cfg.n, cfg.d, cfg.grad_mode, cfg.init_mode = int(n), int(d), int(grad_mode), int(init_mode)
    cfg.A, cfg.labels = _ptr(A), _ptr(labels)
    cfg.shard_offsets = None if so is None else so.ctypes.data_as(C.c_void_p)
    cfg.x0, cfg.grad0 = _ptr(x0), _ptr(grad0)
    cfg.lam, cfg.gamma = float(lam), float(gamma)
    cfg.worker_levels, cfg.m_worker, cfg.zeta_worker = wl, len(list(worker_levels)), float(zeta_worker)
    cfg.master_levels, cfg.m_master, cfg.zeta_master = ml, len(list(master_levels)), float(zeta_master)
    cfg.seed, cfg.flags, cfg.pad = int(seed), int(flags), 0
    cfg.stream = C.c_void_p(int(stream)) if stream else None
    tw, tm = _triggers(worker_triggers, cfg.m_worker), _triggers(master_triggers, cfg.m_master)
    if tw is not None:
        cfg.worker_triggers = tw
    if tm is not None:
        cfg.master_triggers = tm
    keep_csr = None
    if csr is not None:
        rp = np.ascontiguousarray(csr[0], dtype=np.int64)
        ci = np.ascontiguousarray(csr[1], dtype=np.int32)
        cv = None if csr[2] is None else np.ascontiguousarray(csr[2], dtype=np.float32)
        cfg.csr_row_ptr = rp.ctypes.data_as(C.c_void_p)
        cfg.csr_col = ci.ctypes.data_as(C.c_void_p)
        cfg.csr_val = None if cv is None else cv.ctypes.data_as(C.c_void_p)
        keep_csr = (rp, ci, cv)
    return cfg, (wl, ml, so, A, labels, x0, grad0, tw, tm, keep_csr)


def adacgd_workspace_bytes(cfg: Config) -> int:
    lib = load_library()
    out = C.c_int64(0)
    rc = lib.adacgd_workspace_bytes(C.byref(cfg), C.byref(out))
    if rc:
        raise AdaCGDError(rc, lib.adacgd_last_error(None).decode())
    return out.value


def adacgd_init(cfg: Config) -> C.c_void_p:
    lib = load_library()
    ctx = C.c_void_p(None)
    rc = lib.adacgd_init(C.byref(cfg), C.byref(ctx))
    if rc:
        raise AdaCGDError(rc, lib.adacgd_last_error(None).decode())
    return ctx


STATIC_WORKSPACE_BYTES = 64 << 20


def adacgd_init_static(cfg: Config) -> C.c_void_p:
    lib = load_library()
    ctx = C.c_void_p(None)
    rc = lib.adacgd_init_static(C.byref(cfg), C.byref(ctx))
    if rc:
        raise AdaCGDError(rc, lib.adacgd_last_error(None).decode())
    return ctx


def adacgd_step(ctx, ext=None, ext_D=None, nsteps=1):
    lib = load_library()
    rc = lib.adacgd_step(ctx, _ptr(ext), _ptr(ext_D), int(nsteps))
    if rc:
        raise AdaCGDError(rc, lib.adacgd_last_error(ctx).decode())


def adacgd_state(ctx, field, out: np.ndarray):
    """Copies a field into the host array `out` (whose size must match exactly)."""
    lib = load_library()
    rc = lib.adacgd_state(ctx, int(field), out.ctypes.data_as(C.c_void_p), out.nbytes, 0)
    if rc:
        raise AdaCGDError(rc, lib.adacgd_last_error(ctx).decode())
    return out


def adacgd_set_state(ctx, field, src: np.ndarray):
    """Restores a persistent field from the host array `src` (whose size must match exactly)."""
    lib = load_library()
    src = np.ascontiguousarray(src)
    rc = lib.adacgd_set_state(ctx, int(field), src.ctypes.data_as(C.c_void_p), src.nbytes, 0)
    if rc:
        raise AdaCGDError(rc, lib.adacgd_last_error(ctx).decode())


def adacgd_destroy(ctx):
    lib = load_library()
    rc = lib.adacgd_destroy(ctx)
    if rc:
        raise AdaCGDError(rc, "destroy failed")


class AdaCGD:
    """Convenience owner of one context: allocates the workspace with torch, keeps the
    borrowed tensors alive, and shapes the outputs of adacgd_state."""

    def __init__(self, static_workspace=False, **kw):
        """static_workspace: adacgd_init_static instead of adacgd_init (no workspace tensor is made)."""
        import torch
        self.torch = torch
        if not torch.cuda.is_available():
            raise RuntimeError("the AdaCGD engine needs a GPU; there is no CPU path")
        kw.setdefault("stream", torch.cuda.current_stream().cuda_stream)
        self.n, self.d = int(kw["n"]), int(kw["d"])
        self.worker_levels = list(kw["worker_levels"])
        self.master_levels = list(kw.get("master_levels", ()))
        self.grad_mode = kw.get("grad_mode", GRAD_EXTERNAL)
        self.cfg, self._keep = make_config(**kw)
        self.ctx = None
        if static_workspace:
            self.workspace = None
            self.ctx = adacgd_init_static(self.cfg)
        else:
            nbytes = adacgd_workspace_bytes(self.cfg)
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            self.cfg.workspace = C.c_void_p(self.workspace.data_ptr())
            self.cfg.workspace_bytes = nbytes
            self.ctx = adacgd_init(self.cfg)
        self._ext_keep = None

    def step(self, ext=None, ext_D=None, nsteps=1):
        if ext is not None:
            assert ext.is_cuda and ext.dtype == self.torch.float32 and ext.is_contiguous()
            assert ext.numel() == nsteps * self.n * self.d
        if ext_D is not None:
            assert ext_D.is_cuda and ext_D.dtype == self.torch.float64 and ext_D.numel() == nsteps * self.n
        self._ext_keep = (ext, ext_D)
        adacgd_step(self.ctx, ext, ext_D, nsteps)

    def _get(self, field, shape, dtype):
        return adacgd_state(self.ctx, field, np.empty(shape, dtype=dtype))

    def state(self, field):
        n, d = self.n, self.d
        mw, mm = len(self.worker_levels), len(self.master_levels)
        f32, f64, i32, i64, u64 = np.float32, np.float64, np.int32, np.int64, np.uint64
        if field in (F_X, F_G, F_GTILDE, F_GTILDE_PREV):
            return self._get(field, (d,), f32)
        if field in (F_GI, F_PREV_GRAD, F_GRAD):
            return self._get(field, (n, d), f32)
        if field == F_LEVEL:
            return self._get(field, (n,), i32)
        if field in (F_SQNORM, F_D):
            return self._get(field, (n,), f64)
        if field == F_ERR:
            return self._get(field, (n, mw), f64)
        if field == F_MSG_COUNT:
            return self._get(field, (n,), i64)
        if field in (F_MSG_IDX, F_MSG_VAL):
            total = int(self.state(F_MSG_COUNT).sum())
            return self._get(field, (total,), i32 if field == F_MSG_IDX else f32)
        if field == F_M_LEVEL:
            return self._get(field, (1,), i32)
        if field in (F_M_SQNORM, F_M_D):
            return self._get(field, (1,), f64)
        if field == F_M_ERR:
            return self._get(field, (mm,), f64)
        if field == F_M_MSG_COUNT:
            return self._get(field, (1,), i64)
        if field in (F_M_MSG_IDX, F_M_MSG_VAL):
            total = int(self.state(F_M_MSG_COUNT)[0])
            return self._get(field, (total,), i32 if field == F_M_MSG_IDX else f32)
        if field == F_STEP:
            return self._get(field, (1,), i64)
        if field == F_LEVEL_HIST:
            return self._get(field, (mw + 1,), u64)
        if field == F_M_LEVEL_HIST:
            return self._get(field, (mm + 1,), u64)
        if field == F_COMM:
            return self._get(field, (4,), u64)
        if field == F_ESTIMATOR_ERR:
            return self._get(field, (1,), f64)
        if field in (F_REPAIRS, F_CANDIDATES):
            return self._get(field, (2,), u64)
        if field == F_QCODES:
            return self._get(field, (n, d), np.int16)
        if field == F_QSCALE:
            return self._get(field, (n,), f32)
        if field == F_QBSCALE:
            return self._get(field, (n, (d + 63) // 64), f32)
        if field == F_RANK_SPECTRUM:
            cols = [p[1] for k, p in self.worker_levels if k == RANK]
            return self._get(field, (n, cols[0]), f64)
        if field == F_KERNEL_MS:
            return self._get(field, (2, len(KERNELS)), f64)
        raise ValueError(field)

    CHECKPOINT_FIELDS = (F_X, F_G, F_GTILDE, F_GTILDE_PREV, F_GI, F_PREV_GRAD, F_STEP, F_LEVEL_HIST, F_M_LEVEL_HIST)

    def set_state(self, field, array):
        adacgd_set_state(self.ctx, field, array)

    def checkpoint(self):
        """{field: host array} of everything a restored run needs (fields this mode does not keep are left out)."""
        out = {}
        for f in self.CHECKPOINT_FIELDS:
            if f in (F_G, F_M_LEVEL_HIST) and not self.master_levels:
                continue
            if f == F_PREV_GRAD and self.grad_mode == DIFF_EXTERNAL:
                continue
            out[f] = self.state(f)
        return out

    def restore(self, ckpt):
        for f, a in ckpt.items():
            self.set_state(f, a)

    def messages(self):
        """Per-worker (indices, values) of the last step's Top-K messages."""
        cnt = self.state(F_MSG_COUNT)
        idx, val = self.state(F_MSG_IDX), self.state(F_MSG_VAL)
        off = np.concatenate([[0], np.cumsum(cnt)])
        return [(idx[off[i]:off[i + 1]], val[off[i]:off[i + 1]]) for i in range(self.n)]

    def kernel_ms(self):
        """{kernel: (total ms, launches)} since the last call (needs FLAG_KERNEL_TIMING)."""
        a = self.state(F_KERNEL_MS)
        return {k: (float(a[0, i]), int(a[1, i])) for i, k in enumerate(KERNELS)}

    def close(self):
        if self.ctx is not None:
            adacgd_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
