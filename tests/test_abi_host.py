"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad configurations with the documented codes."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2211_00188_amd import engine as E

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

pytestmark = pytest.mark.skipif(not os.path.exists(E.LIB_PATH), reason="libadacgd.so not built")


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "adacgd.h")).read()
    declared = set(re.findall(r"^(?:int|const char\*)\s+(adacgd_\w+)\s*\(", hdr, flags=re.M))
    assert declared == set(E.EXPORTS)
    lib = E.load_library()
    for name in declared:
        assert getattr(lib, name) is not None


def _cfg(**kw):
    base = dict(n=4, d=100, worker_levels=[(E.TOPK, 1), (E.TOPK, 10)], zeta_worker=1.0,
                master_levels=[(E.TOPK, 5)], zeta_master=0.0, grad_mode=E.GRAD_EXTERNAL)
    base.update(kw)
    return E.make_config(**base)


def test_new_level_kinds_are_accepted():
    base = E.adacgd_workspace_bytes(_cfg(d=4096)[0])
    blk = E.adacgd_workspace_bytes(_cfg(d=4096, worker_levels=[(E.TOPK, 4), (E.QUANT_BLOCK, (4, 256))])[0])
    rnk = E.adacgd_workspace_bytes(_cfg(d=4096, worker_levels=[(E.RANK, (1, 16)), (E.RANK, (8, 16)), (E.TOPK, 4096)])[0])
    assert blk > base and rnk > base


def test_workspace_size_is_reported_and_grows_with_problem():
    a = E.adacgd_workspace_bytes(_cfg()[0])
    b = E.adacgd_workspace_bytes(_cfg(n=8, d=100000)[0])
    assert 0 < a < b
    assert a % 256 == 0


@pytest.mark.parametrize("kw,code", [
    (dict(n=0), 1), (dict(d=0), 1), (dict(d=1 << 31), 1), (dict(n=70000), 1),
    (dict(worker_levels=[(E.TOPK, 0)]), 1), (dict(worker_levels=[(E.TOPK, 101)]), 1),
    (dict(worker_levels=[(E.QUANT, 1)]), 1), (dict(worker_levels=[(E.QUANT, 17)]), 1),
    (dict(worker_levels=[]), 1), (dict(worker_levels=[(7, 3)]), 1),
    (dict(zeta_worker=-1.0), 1), (dict(zeta_worker=float("nan")), 1), (dict(gamma=float("inf")), 1),
    (dict(worker_levels=[(E.TOPK, 10), (E.TOPK, 1)]), 2),
    (dict(worker_levels=[(E.TOPK, 50), (E.QUANT, 2)]), 2),
    (dict(grad_mode=E.DIFF_EXTERNAL, init_mode=E.INIT_FULLGRAD), 1),
    (dict(grad_mode=5), 1),
    (dict(init_mode=3), 1),
    (dict(init_mode=E.INIT_COMPRESSED, worker_levels=[(E.TOPK, 1), (E.QUANT, 8)]), 1),
    (dict(worker_triggers=[(1.0, 0.0), (1.0, -0.1)]), 1),
    (dict(worker_triggers=[(float("inf"), 0.0), (1.0, 0.0)]), 1),
    (dict(master_triggers=[(0.0, float("nan"))]), 1),
    (dict(worker_levels=[(E.QUANT_BLOCK, (4, 100))]), 1),          # block length not a power of two
    (dict(worker_levels=[(E.QUANT_BLOCK, (4, 32))]), 1), (dict(worker_levels=[(E.QUANT_BLOCK, (4, 4096))]), 1),
    (dict(worker_levels=[(E.QUANT_BLOCK, (1, 64))]), 1),
    (dict(worker_levels=[(E.RANK, (2, 16))]), 1),                  # d = 100 is not a multiple of 16
    (dict(d=512, worker_levels=[(E.RANK, (2, 8))]), 1), (dict(d=512, worker_levels=[(E.RANK, (17, 16))]), 1),
    (dict(d=512, worker_levels=[(E.RANK, (2, 32))]), 1),           # fewer rows than columns
    (dict(d=4096, worker_levels=[(E.RANK, (2, 16)), (E.RANK, (4, 32))]), 1),   # two column counts
    (dict(d=512, worker_levels=[(E.RANK, (8, 16)), (E.RANK, (2, 16))]), 2),    # alpha = K/c not ascending
])
def test_bad_configurations_are_rejected(kw, code):
    with pytest.raises(E.AdaCGDError) as ei:
        E.adacgd_workspace_bytes(_cfg(**kw)[0])
    assert ei.value.code == code
    assert str(ei.value)


def test_unsorted_levels_accepted_with_flag():
    cfg, _ = _cfg(worker_levels=[(E.TOPK, 10), (E.TOPK, 1)], flags=E.FLAG_ANY_LEVEL_ORDER)
    assert E.adacgd_workspace_bytes(cfg) > 0


def test_init_rejects_missing_pointers_without_touching_the_device():
    cfg, _ = _cfg()
    lib = E.load_library()
    ctx = C.c_void_p(None)
    assert lib.adacgd_init(C.byref(cfg), C.byref(ctx)) == 1      # x0 is null
    assert b"x0" in lib.adacgd_last_error(None)
    assert lib.adacgd_destroy(None) == 0
    assert lib.adacgd_step(None, None, None, 1) == 1
    assert lib.adacgd_set_state(None, 0, None, 0, 0) == 1


def test_logistic_shards_validated():
    so = np.array([0, 10, 10, 30, 40], dtype=np.int64)
    with pytest.raises(E.AdaCGDError) as ei:
        E.adacgd_workspace_bytes(_cfg(grad_mode=E.GRAD_LOGISTIC, shard_offsets=so)[0])
    assert ei.value.code == 1 and "empty shard" in str(ei.value)


def test_triggers_replace_the_zeta_argument():
    # with a trigger array the scalar is not read, so an invalid scalar is not an error
    cfg, _ = _cfg(zeta_worker=-1.0, worker_triggers=[(1.0, 0.0), (0.5, 0.1)])
    assert E.adacgd_workspace_bytes(cfg) > 0
    with pytest.raises(ValueError):
        _cfg(worker_triggers=[(1.0, 0.0)])           # one pair per cascade position


def _csr_cfg(row_ptr, col, val=None, d=6, n=2, offsets=(0, 2, 3)):
    return _cfg(n=n, d=d, worker_levels=[(E.TOPK, 1)], master_levels=[], grad_mode=E.GRAD_LOGISTIC_CSR,
                shard_offsets=np.array(offsets, dtype=np.int64), csr=(row_ptr, col, val))


def test_sparse_rows_are_validated_on_the_host():
    ok = _csr_cfg([0, 2, 2, 4], [1, 5, 0, 3])
    assert E.adacgd_workspace_bytes(ok[0]) > 0
    with_values = _csr_cfg([0, 2, 2, 4], [1, 5, 0, 3], [0.5, -1, 2, 3])
    assert E.adacgd_workspace_bytes(with_values[0]) > E.adacgd_workspace_bytes(ok[0])
    for row_ptr, col, what in [
        ([1, 2, 2, 4], [1, 5, 0, 3], "row_ptr[0]"),
        ([0, 2, 1, 4], [1, 5, 0, 3], "decreases"),
        ([0, 2, 2, 4], [1, 6, 0, 3], "columns"),        # column == d
        ([0, 2, 2, 4], [1, 5, 0, -1], "columns"),
        ([0, 2, 2, 4], [5, 1, 0, 3], "columns"),        # not ascending
        ([0, 2, 2, 4], [1, 1, 0, 3], "columns"),        # duplicate
    ]:
        with pytest.raises(E.AdaCGDError) as ei:
            E.adacgd_workspace_bytes(_csr_cfg(row_ptr, col)[0])
        assert ei.value.code == 1 and what in str(ei.value), (row_ptr, col, str(ei.value))
    cfg, _ = _cfg(grad_mode=E.GRAD_LOGISTIC_CSR, shard_offsets=np.array([0, 1, 2, 3, 4], dtype=np.int64))
    with pytest.raises(E.AdaCGDError):
        E.adacgd_workspace_bytes(cfg)               # no row_ptr


def test_header_is_plain_c_and_matches_the_binding(tmp_path):
    """The header compiles as C99 on its own, and the configuration struct has the size and field
    offsets the ctypes binding assumes."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    fields = [name for name, _ in E.Config._fields_]
    renamed = {"lam": "lambda"}
    src = tmp_path / "abi.c"
    src.write_text(
        '#include <stdio.h>\n#include <stddef.h>\n#include "adacgd.h"\n'
        "int main(void) {\n"
        '  printf("%zu %zu %zu\\n", sizeof(adacgd_config), sizeof(adacgd_level), sizeof(adacgd_trigger));\n'
        + "".join('  printf("%%zu\\n", offsetof(adacgd_config, %s));\n' % renamed.get(f, f) for f in fields)
        + "  return (int)(ADACGD_NUM_KERNELS - %d + ADACGD_F_ESTIMATOR_ERR - %d + ADACGD_F_RANK_SPECTRUM - %d"
          " + ADACGD_RANK - %d);\n}\n" % (len(E.KERNELS), E.F_ESTIMATOR_ERR, E.F_RANK_SPECTRUM, E.RANK))
    exe = tmp_path / "abi"
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert [int(v) for v in out[:3]] == [C.sizeof(E.Config), C.sizeof(E.Level), C.sizeof(E.Trigger)]
    assert [int(v) for v in out[3:]] == [getattr(E.Config, f).offset for f in fields]
