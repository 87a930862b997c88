"""Host-only checks of the boundary: the built library exports every entry point that
include/abs.h declares, and the pure-host parts of it behave (no GPU call is made)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2406_13936_amd", "libabs.so")


def _declared():
    src = open(os.path.join(ROOT, "include", "abs.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"\b(abs_[a-z0-9_]+)\s*\(", src)
    return sorted(set(names))


def _lib():
    if not os.path.exists(LIB):
        import __graft_entry__ as g
        g.build()
    return C.CDLL(LIB)


def test_every_declared_entry_point_is_exported():
    names = _declared()
    assert "abs_local_step" in names and "abs_average_replicas" in names and len(names) >= 15
    lib = _lib()
    for n in names:
        assert hasattr(lib, n), n


def test_header_is_plain_c():
    """The boundary is a C ABI: the header must compile as C99 with no C++ in it."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler here")
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c",
                        os.path.join(ROOT, "include", "abs.h")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_binding_lists_the_same_entry_points():
    from paper_2406_13936_amd import binding
    assert sorted(binding.EXPORTS) == _declared()


def test_batch_size_rule_on_the_host():
    from paper_2406_13936_amd import binding as B
    B.load_library()
    rs = []
    for T in (5, 40, 17):
        r = B.TestResult()
        r.T = T
        rs.append(r)
    assert B.next_batch_size(rs, [16, 16, 16], 512, sync_max=True) == [40, 40, 40]
    assert B.next_batch_size(rs, [16, 16, 16], 512, sync_max=False) == [16, 40, 17]
    assert B.next_batch_size(rs, [16, 16, 16], 32, sync_max=True) == [32, 32, 32]
    rs[1].T = -3
    assert B.next_batch_size(rs, [16, 16, 16], 512, sync_max=False) == [16, 16, 17]


def test_config_validation_without_a_gpu():
    from paper_2406_13936_amd import binding as B
    lib = B.load_library()
    dims = (C.c_int * 3)(20, 16, 4)          # 20 is not a multiple of 8
    cfg = B._Config(2, dims, 1, 1, B.PREC_BF16, 2, 64, 0, 0, 0.9, 0.999, 1e-8, 0, 1, None, None, 0)
    n = C.c_size_t(0)
    assert lib.abs_workspace_bytes(C.byref(cfg), 100, C.byref(n)) == 5      # ABS_EUNSUPPORTED
    assert b"multiples of 8" in lib.abs_last_error(None)
    cfg.prec = B.PREC_F32
    assert lib.abs_workspace_bytes(C.byref(cfg), 100, C.byref(n)) == 0 and n.value > 0
    p = C.c_int64(0)
    assert lib.abs_n_params(C.byref(cfg), C.byref(p)) == 0
    assert p.value == 20 * 16 + 16 + 16 * 4 + 4
    cfg.b_cap = 1
    assert lib.abs_workspace_bytes(C.byref(cfg), 100, C.byref(n)) == 1      # ABS_EINVAL


def test_lr_schedule_matches_oracle_on_the_host():
    from paper_2406_13936_amd import binding as B
    from oracle import abs_oracle as O
    for s in (0, 1, 49, 50, 51, 300, 999, 1000, 1200):
        assert B.lr_schedule(s, 1000, 50, 0.05, 0.005) == pytest.approx(O.lr_schedule(s, 1000, 50, 0.05, 0.005),
                                                                         rel=1e-14)
    with pytest.raises(B.AbsError):
        B.lr_schedule(3, 10, 20, 0.1, 0.01)


def test_linear_lr_scaling_on_the_host():
    from paper_2406_13936_amd import binding as B
    assert B.lr_linear_scaling(0.05, 2048, 256) == pytest.approx(0.4)
    with pytest.raises(B.AbsError):
        B.lr_linear_scaling(0.05, 0, 256)


def test_null_context_is_rejected_by_every_stepping_entry_point():
    from paper_2406_13936_amd import binding as B
    lib = B.load_library()
    lib.abs_local_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_float]
    assert lib.abs_local_step(None, None, 4, C.c_float(0.1)) == 1                     # ABS_EINVAL
    assert lib.abs_local_step_ragged(None, None, 4, None, C.c_float(0.1)) == 1
    assert lib.abs_local_step_accumulated(None, None, 8, 4, C.c_float(0.1)) == 1
    assert lib.abs_norm_test(None, 0.5, None) == 1
    assert lib.abs_norm_test_per_worker(None, None, None) == 1
    assert lib.abs_norm_test_fpc(None, 0.5, 10, None) == 1
    assert lib.abs_average_replicas(None) == 1
    assert b"NULL" in lib.abs_last_error(None)
