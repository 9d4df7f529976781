"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and its argument validation answers with the documented error codes before any
device work is attempted."""
import ctypes as C
import os
import re

import pytest

import paper_2203_16340_amd as L

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "lbfgsb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lbfgsb_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert len(names) >= 18 and "lbfgsb_create" in names and "lbfgsb_step" in names
    lib = L.lib()
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in include/lbfgsb.h but not exported"
    assert sorted(L.EXPORTS) == names            # the Python binding covers the same names


def test_struct_layouts_match_the_header(tmp_path):
    """sizeof/offsetof as gcc sees include/lbfgsb.h against the ctypes mirrors: guards against a
    field added or reordered on one side only."""
    import subprocess
    src = tmp_path / "sz.c"
    src.write_text(
        '#include <stdio.h>\n#include <stddef.h>\n#include "lbfgsb.h"\n'
        'int main(void){printf("%zu %zu %zu %zu %zu %zu %zu\\n", sizeof(lbfgsb_objective), sizeof(lbfgsb_options),'
        ' sizeof(lbfgsb_info), offsetof(lbfgsb_objective, lambda), offsetof(lbfgsb_options, a_pass),'
        ' offsetof(lbfgsb_info, n_fixed), offsetof(lbfgsb_info, gp)); return 0;}\n')
    exe = tmp_path / "sz"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    got = [int(t) for t in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert got == [C.sizeof(L.Objective), C.sizeof(L.Options), C.sizeof(L.Info), L.Objective.lam.offset,
                   L.Options.a_pass.offset, L.Info.n_fixed.offset, L.Info.gp.offset]


def test_auglag_struct_layouts_and_argument_checks(tmp_path):
    import subprocess
    src = tmp_path / "sz2.c"
    src.write_text(
        '#include <stdio.h>\n#include <stddef.h>\n#include "lbfgsb.h"\n'
        'int main(void){printf("%zu %zu %zu %zu %zu\\n", sizeof(lbfgsb_auglag_options), sizeof(lbfgsb_auglag_info),'
        ' offsetof(lbfgsb_auglag_info, violation), offsetof(lbfgsb_objective, n_extra),'
        ' offsetof(lbfgsb_objective, extra_weight)); return 0;}\n')
    exe = tmp_path / "sz2"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    got = [int(t) for t in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert got == [C.sizeof(L.AuglagOptions), C.sizeof(L.AuglagInfo), L.AuglagInfo.violation.offset,
                   L.Objective.n_extra.offset, L.Objective.extra_weight.offset]
    lib = L.lib()
    ao = L.AuglagOptions()
    lib.lbfgsb_auglag_default_options(C.byref(ao))
    assert (ao.rho0, ao.ctol, ao.max_outer) == (1.0, 1e-8, 100)
    o = L.default_options()
    stacked = _obj(rows=203, cols=100)
    plain = lib.lbfgsb_workspace_bytes(100, 5, C.byref(stacked), C.byref(o))
    assert lib.lbfgsb_auglag_workspace_bytes(100, 5, C.byref(stacked), 3, C.byref(o)) > plain
    assert lib.lbfgsb_auglag_workspace_bytes(100, 5, C.byref(stacked), 203, C.byref(o)) == 0      # no data row left
    assert lib.lbfgsb_auglag_workspace_bytes(100, 5, C.byref(_obj(kind=2, rows=203)), 3, C.byref(o)) == 0
    assert lib.lbfgsb_auglag_rows_workspace_bytes(100, 5, C.byref(_obj()), 3, C.byref(o)) > plain - 203 * 8 * 3
    assert lib.lbfgsb_auglag_rows_workspace_bytes(100, 5, C.byref(_obj()), 65, C.byref(o)) == 0   # at most 64 separate rows
    assert lib.lbfgsb_auglag_rows_workspace_bytes(100, 5, C.byref(_obj(kind=2)), 1, C.byref(o)) == 0
    # the quadratic form needs a square matrix
    assert lib.lbfgsb_workspace_bytes(100, 5, C.byref(_obj(kind=3, rows=100, cols=100)), C.byref(o)) > 0
    assert lib.lbfgsb_workspace_bytes(100, 5, C.byref(_obj(kind=3, rows=200, cols=100)), C.byref(o)) == 0
    h = C.c_void_p()
    assert lib.lbfgsb_auglag_create(C.byref(h), 100, 5, 0x3000, 0x4000, C.byref(stacked), -1, C.byref(o), C.byref(ao),
                                    0x10000, 1 << 24, None) == L.E_INVALID_ARG
    assert lib.lbfgsb_auglag_solve(None, None, None) == L.E_INVALID_ARG
    lib.lbfgsb_auglag_destroy(None)


def test_transport_kinds_argument_checks():
    """The matrix-variable kinds: n = rows*cols, lambda > 0, no extra rows; the marginal-constraint entry point takes
    these kinds only.  No device call is reached."""
    lib = L.lib()
    o = L.default_options()
    ao = L.AuglagOptions()
    lib.lbfgsb_auglag_default_options(C.byref(ao))

    def ot(kind=L.OBJ_OT_GAUSS, rows=30, cols=20, lam=0.5, n_extra=0):
        return L.Objective(kind, 0, rows, cols, cols, 0x1000, None, lam, 0.0, None, None, n_extra, None, None, None)

    plain = lib.lbfgsb_workspace_bytes(600, 5, C.byref(ot()), C.byref(o))
    assert plain > 2 * 5 * 600 * 8
    assert lib.lbfgsb_workspace_bytes(600, 5, C.byref(ot(kind=L.OBJ_OT_ENTROPY)), C.byref(o)) == plain
    assert lib.lbfgsb_workspace_bytes(20, 5, C.byref(ot()), C.byref(o)) == 0            # n is rows*cols, not cols
    assert lib.lbfgsb_workspace_bytes(600, 5, C.byref(ot(lam=0.0)), C.byref(o)) == 0
    assert b"lambda" in lib.lbfgsb_last_error()
    assert lib.lbfgsb_workspace_bytes(600, 5, C.byref(ot(n_extra=1)), C.byref(o)) == 0
    # long vectors take the other Gram kernels, whose partials are laid out differently: still a valid size
    big = lib.lbfgsb_workspace_bytes(1000 * 1000, 10, C.byref(ot(rows=1000, cols=1000)), C.byref(o))
    assert big > 2 * 10 * 10**6 * 8 and big % 256 == 0
    assert lib.lbfgsb_workspace_bytes(1000 * 1000, 20, C.byref(ot(rows=1000, cols=1000)), C.byref(o)) > big
    with_al = lib.lbfgsb_auglag_marginals_workspace_bytes(5, C.byref(ot()), C.byref(o))
    assert with_al >= plain + 3 * 50 * 8
    assert lib.lbfgsb_auglag_marginals_workspace_bytes(5, C.byref(_obj()), C.byref(o)) == 0       # least squares: wrong kind
    h = C.c_void_p()
    rc = lib.lbfgsb_auglag_create_marginals(C.byref(h), 5, 0x3000, 0x4000, C.byref(_obj()), 0x5000, C.byref(o), C.byref(ao),
                                            0x10000, 1 << 24, None)
    assert rc == L.E_INVALID_ARG and not h
    rc = lib.lbfgsb_auglag_create_marginals(C.byref(h), 5, 0x3000, 0x4000, C.byref(ot()), None, C.byref(o), C.byref(ao),
                                            0x10000, 1 << 24, None)
    assert rc == L.E_INVALID_ARG
    rc = lib.lbfgsb_auglag_create_marginals(C.byref(h), 5, 0x3000, 0x4000, C.byref(ot()), 0x5000, C.byref(o), C.byref(ao),
                                            0x10000, 64, None)
    assert rc == L.E_INVALID_ARG and b"too small" in lib.lbfgsb_last_error()


def test_history_record_layout_matches_the_header(tmp_path):
    import subprocess
    src = tmp_path / "sz3.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "lbfgsb.h"\n'
                   'int main(void){printf("%zu %zu %zu %d\\n", sizeof(lbfgsb_iter_record), offsetof(lbfgsb_iter_record, alpha),'
                   ' offsetof(lbfgsb_iter_record, memory_resets), LBFGSB_HISTORY_CAPACITY); return 0;}\n')
    exe = tmp_path / "sz3"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    got = [int(t) for t in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert got == [C.sizeof(L.IterRecord), L.IterRecord.alpha.offset, L.IterRecord.memory_resets.offset, L.HISTORY_CAPACITY]
    cnt = C.c_int(7)
    assert L.lib().lbfgsb_get_history(None, None, 0, C.byref(cnt)) == L.E_INVALID_ARG


def test_default_options():
    o = L.default_options()
    assert (o.eps, o.armijo_c1, o.backtrack, o.max_backtracks) == (1e-10, 1e-4, 0.5, 60)
    assert (o.tol, o.tol_relative, o.max_iter, o.refresh_every, o.poll_every, o.a_pass) == (1e-8, 0, 1000, 32, 8, 0)


def _obj(kind=0, dtype=0, rows=200, cols=100, ld=None, A=0x1000, b=0x2000):
    return L.Objective(kind, dtype, rows, cols, cols if ld is None else ld, A, b, 0.0, 0.0)


def test_workspace_bytes_validates_and_scales():
    lib = L.lib()
    o = L.default_options()
    base = lib.lbfgsb_workspace_bytes(100, 5, C.byref(_obj()), C.byref(o))
    assert base > 0 and base % 256 == 0
    # room for 2*m*n doubles of pair memory at least
    assert base >= 2 * 5 * 100 * 8
    assert lib.lbfgsb_workspace_bytes(100, 10, C.byref(_obj()), C.byref(o)) > base
    for bad in [dict(n=0), dict(n=101), dict(m=0), dict(m=32), dict(kind=7), dict(dtype=3), dict(rows=0), dict(ld=99)]:
        n = bad.pop("n", 100)
        m = bad.pop("m", 5)
        assert lib.lbfgsb_workspace_bytes(n, m, C.byref(_obj(**bad)), C.byref(o)) == 0
        assert lib.lbfgsb_last_error()
    # the split objective has 2*cols variables
    assert lib.lbfgsb_workspace_bytes(200, 5, C.byref(_obj(kind=1)), C.byref(o)) > 0
    assert lib.lbfgsb_workspace_bytes(100, 5, C.byref(_obj(kind=1)), C.byref(o)) == 0


def test_create_rejects_bad_arguments_before_touching_the_device():
    lib = L.lib()
    h = C.c_void_p()
    o = L.default_options()
    obj = _obj()
    ws = 0x10000
    rc = lib.lbfgsb_create(C.byref(h), 100, 5, None, 0x3000, C.byref(obj), C.byref(o), ws, 1 << 20, None)
    assert rc == L.E_INVALID_ARG and not h
    rc = lib.lbfgsb_create(C.byref(h), 100, 0, 0x3000, 0x4000, C.byref(obj), C.byref(o), ws, 1 << 20, None)
    assert rc == L.E_INVALID_ARG
    rc = lib.lbfgsb_create(C.byref(h), 100, 5, 0x3000, 0x4000, C.byref(obj), C.byref(o), ws + 8, 1 << 20, None)
    assert rc == L.E_INVALID_ARG and b"aligned" in lib.lbfgsb_last_error()
    rc = lib.lbfgsb_create(C.byref(h), 100, 5, 0x3000, 0x4000, C.byref(obj), C.byref(o), ws, 16, None)
    assert rc == L.E_INVALID_ARG and b"too small" in lib.lbfgsb_last_error()
    bad = L.default_options(backtrack=1.5)
    rc = lib.lbfgsb_create(C.byref(h), 100, 5, 0x3000, 0x4000, C.byref(obj), C.byref(bad), ws, 1 << 20, None)
    assert rc == L.E_INVALID_ARG
    rc = lib.lbfgsb_create(None, 100, 5, 0x3000, 0x4000, C.byref(obj), C.byref(o), ws, 1 << 20, None)
    assert rc == L.E_INVALID_ARG
    # NULL solver handles are errors, never crashes; destroy(NULL) is a no-op
    assert lib.lbfgsb_step(None, None) == L.E_INVALID_ARG
    assert lib.lbfgsb_solve(None, None) == L.E_INVALID_ARG
    assert lib.lbfgsb_set_x(None, None) == L.E_INVALID_ARG
    assert lib.lbfgsb_get_info(None, None) == L.E_INVALID_ARG
    lib.lbfgsb_destroy(None)


def test_product_path_does_not_reach_the_oracle():
    """The binding and the HIP sources never import, include or link anything under oracle/."""
    pkg = os.path.join(ROOT, "paper_2203_16340_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in text.replace("no fallback", ""), f"{fn} mentions the oracle"


def test_benchmark_refuses_more_than_one_gpu_and_a_machine_without_one():
    """bench.py measures one GPU: --gpus N > 1 ends with a message that says so; without a GPU it ends with an
    error instead of measuring anything else."""
    import subprocess
    import sys
    import torch
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=300)
    assert r.returncode != 0 and "ONE GPU" in (r.stdout + r.stderr)
    if not torch.cuda.is_available():
        r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--config", "C1"], capture_output=True, text=True,
                           timeout=300)
        assert r.returncode != 0 and "no GPU" in (r.stdout + r.stderr)
        assert '"metric"' not in r.stdout
