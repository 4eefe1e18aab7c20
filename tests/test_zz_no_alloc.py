"""adacgd_init_static -- the entry point for callers that cannot allocate device memory -- against
adacgd_init with a caller-provided workspace, through the C ABI: every state vector, level and message
bit for bit, on two contexts in a row that share the library's static device array, the second one
smaller than the first (so that it runs on what the first left behind)."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOPK, QUANT, QUANT_BLOCK, RANK = 0, 1, 2, 3


def _run(E, torch, static, n, d, levels, master, mode, steps, seed):
    """Drives one context through the C entry points only; returns every field worth comparing."""
    lib = E.load_library()
    rng = np.random.default_rng(seed)
    host = [rng.standard_normal((n, d)).astype(np.float32)]
    for t in range(steps):
        host.append((host[-1] + np.float32(10.0 ** rng.uniform(-2, 0)) * rng.standard_normal((n, d))).astype(np.float32))
    dev = [torch.from_numpy(h).cuda() for h in host]
    Ds = [torch.from_numpy(np.sum(h.astype(np.float64) ** 2, axis=1) * rng.uniform(0.05, 2.0, n)).cuda() for h in host]
    x0 = torch.from_numpy(rng.standard_normal(d).astype(np.float32)).cuda()
    diff = mode == E.DIFF_EXTERNAL
    cfg, keep = E.make_config(n=n, d=d, gamma=0.05, worker_levels=levels, zeta_worker=0.8, master_levels=master,
                              zeta_master=0.0, grad_mode=mode, init_mode=E.INIT_ZERO if diff else E.INIT_FULLGRAD,
                              x0=x0, grad0=None if diff else dev[0], seed=99, flags=E.FLAG_ANY_LEVEL_ORDER,
                              stream=torch.cuda.current_stream().cuda_stream)
    need = C.c_int64(0)
    assert lib.adacgd_workspace_bytes(C.byref(cfg), C.byref(need)) == 0
    ctx = C.c_void_p(None)
    ws = None
    if static:
        assert need.value <= E.STATIC_WORKSPACE_BYTES
        rc = lib.adacgd_init_static(C.byref(cfg), C.byref(ctx))
    else:
        ws = torch.empty(need.value, dtype=torch.uint8, device="cuda")
        cfg.workspace, cfg.workspace_bytes = C.c_void_p(ws.data_ptr()), need.value
        rc = lib.adacgd_init(C.byref(cfg), C.byref(ctx))
    assert rc == 0, lib.adacgd_last_error(None)

    def field(f, shape, dtype):
        out = np.empty(shape, dtype=dtype)
        rc = lib.adacgd_state(ctx, f, out.ctypes.data_as(C.c_void_p), out.nbytes, 0)
        assert rc == 0, (f, lib.adacgd_last_error(ctx))
        return out

    got = []
    for t in range(1, steps + 1):
        rc = lib.adacgd_step(ctx, C.c_void_p(dev[t].data_ptr()), C.c_void_p(Ds[t].data_ptr()) if diff else None, 1)
        assert rc == 0, lib.adacgd_last_error(ctx)
        cnt = field(E.F_MSG_COUNT, (n,), np.int64)
        tot = int(cnt.sum())
        got.append([field(E.F_LEVEL, (n,), np.int32), cnt, field(E.F_MSG_IDX, (tot,), np.int32),
                    field(E.F_MSG_VAL, (tot,), np.float32), field(E.F_X, (d,), np.float32),
                    field(E.F_G, (d,), np.float32), field(E.F_GTILDE, (d,), np.float32),
                    field(E.F_GI, (n, d), np.float32), field(E.F_SQNORM, (n,), np.float64),
                    field(E.F_ERR, (n, len(levels)), np.float64), field(E.F_M_LEVEL, (1,), np.int32),
                    field(E.F_LEVEL_HIST, (len(levels) + 1,), np.uint64)])
    assert lib.adacgd_destroy(ctx) == 0
    del ws
    return got


def _same(a, b, tag):
    assert len(a) == len(b)
    for t, (sa, sb) in enumerate(zip(a, b)):
        for k, (fa, fb) in enumerate(zip(sa, sb)):
            assert fa.shape == fb.shape, (tag, t, k)
            assert np.array_equal(fa.view(np.uint8), fb.view(np.uint8)), (tag, t, k)     # NaN patterns included


def test_static_workspace_entry_point_matches_adacgd_init():
    import torch
    from paper_2211_00188_amd import engine as E
    lib = E.load_library()
    big = dict(n=4, d=20 * 8192 + 516, levels=[(TOPK, 30), (QUANT, 4), (TOPK, 2000), (TOPK, 40000)],
               master=[(TOPK, 1500)], mode=E.GRAD_EXTERNAL, steps=3, seed=1)
    small = dict(n=2, d=5003, levels=[(TOPK, 5), (TOPK, 300), (QUANT, 8)], master=[(TOPK, 100)],
                 mode=E.DIFF_EXTERNAL, steps=3, seed=2)
    tiny = dict(n=3, d=700, levels=[(TOPK, 3), (TOPK, 80)], master=[(TOPK, 20)], mode=E.GRAD_EXTERNAL, steps=2, seed=3)
    kinds = dict(n=3, d=16 * 900, levels=[(RANK, (2, 16)), (TOPK, 50), (QUANT_BLOCK, (4, 128)), (TOPK, 1500)],
                 master=[(TOPK, 200)], mode=E.DIFF_EXTERNAL, steps=2, seed=4)
    # two calls in a row on the one array, the second with a smaller input, then one on the one-block path and
    # one with block-wise quantiser and Rank-K levels
    for name, kw in (("big", big), ("small", small), ("tiny", tiny), ("kinds", kinds)):
        got = _run(E, torch, True, **kw)
        ref = _run(E, torch, False, **kw)
        _same(got, ref, name)
        assert any((s[0] > 0).any() for s in ref), name           # something was sent

    # limits: too large for the array, unsupported modes and flags, one context per device at a time
    x0 = torch.zeros(1 << 22, dtype=torch.float32, device="cuda")
    g0 = torch.zeros((4, 1 << 22), dtype=torch.float32, device="cuda")
    cfg, keep = E.make_config(n=4, d=1 << 22, worker_levels=[(TOPK, 100)], zeta_worker=1.0, grad_mode=E.GRAD_EXTERNAL,
                              x0=x0, grad0=g0)
    ctx = C.c_void_p(None)
    assert lib.adacgd_init_static(C.byref(cfg), C.byref(ctx)) == 3 and not ctx.value
    msg = lib.adacgd_last_error(None).decode()
    assert "static workspace holds %d" % E.STATIC_WORKSPACE_BYTES in msg, msg
    x0 = torch.zeros(100, dtype=torch.float32, device="cuda")
    g0 = torch.zeros((2, 100), dtype=torch.float32, device="cuda")
    for bad in (dict(flags=E.FLAG_OVERLAP), dict(flags=E.FLAG_KERNEL_TIMING), dict(grad_mode=E.GRAD_LOGISTIC)):
        kw = dict(n=2, d=100, worker_levels=[(TOPK, 10)], zeta_worker=1.0, grad_mode=E.GRAD_EXTERNAL, x0=x0, grad0=g0)
        kw.update(bad)
        cfg, keep = E.make_config(**kw)
        assert lib.adacgd_init_static(C.byref(cfg), C.byref(ctx)) == 5, bad
    cfg, keep = E.make_config(n=2, d=100, worker_levels=[(TOPK, 10)], zeta_worker=1.0, grad_mode=E.GRAD_EXTERNAL,
                              x0=x0, grad0=g0)
    first, second = C.c_void_p(None), C.c_void_p(None)
    assert lib.adacgd_init_static(C.byref(cfg), C.byref(first)) == 0
    assert lib.adacgd_init_static(C.byref(cfg), C.byref(second)) == 5 and not second.value
    assert "in use" in lib.adacgd_last_error(None).decode()
    assert lib.adacgd_step(first, C.c_void_p(g0.data_ptr()), None, 2) == 0
    assert lib.adacgd_destroy(first) == 0
    assert lib.adacgd_init_static(C.byref(cfg), C.byref(second)) == 0        # free again after destroy
    assert lib.adacgd_destroy(second) == 0
