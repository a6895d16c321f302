"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, and rejects bad arguments before touching a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2204_07104_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ftk.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ftk_[a-z_]+)\s*\(", text)))


def test_header_and_binding_list_the_same_symbols():
    assert declared_functions() == sorted(binding.SYMBOLS)


def test_library_exports_every_declared_symbol():
    L = binding.load()
    for name in declared_functions():
        assert getattr(L, name) is not None


def _create(order, dims, nnz, idx_ptrs, vals_ptr, J, R, flags=0):
    L = binding.load()
    ctx = C.c_void_p(None)
    dims_a = np.asarray(dims, dtype=np.int64)
    J_a = np.asarray(J, dtype=np.int32)
    arr = (C.c_void_p * max(1, len(idx_ptrs)))(*idx_ptrs)
    rc = L.ftk_create(C.byref(ctx), order, dims_a.ctypes.data, nnz, C.cast(arr, C.c_void_p), vals_ptr,
                      J_a.ctypes.data, R, 1, flags)
    return rc, ctx, L.ftk_last_error(None).decode()


def test_create_rejects_bad_arguments_without_a_device():
    i0 = np.zeros(4, dtype=np.int32)
    v = np.ones(4, dtype=np.float32)
    good = dict(order=2, dims=(3, 3), nnz=4, idx_ptrs=[i0.ctypes.data, i0.ctypes.data], vals_ptr=v.ctypes.data,
                J=(2, 2), R=2)
    cases = [
        dict(good, order=0), dict(good, order=11), dict(good, nnz=0), dict(good, nnz=1 << 32),
        dict(good, dims=(0, 3)), dict(good, dims=(3, 1 << 31)), dict(good, J=(0, 2)), dict(good, R=0),
        dict(good, idx_ptrs=[i0.ctypes.data, None]), dict(good, vals_ptr=None), dict(good, flags=8),
    ]
    for kw in cases:
        rc, ctx, msg = _create(**kw)
        assert rc == binding.FTK_EINVAL, (kw, rc, msg)
        assert not ctx.value
        assert msg


def test_null_context_is_rejected_everywhere():
    L = binding.load()
    d = C.c_double(0.0)
    assert L.ftk_sample(None, 1, 1) == binding.FTK_EINVAL
    assert L.ftk_sgd_step(None, 0.0, 0.0, 0.0, 0.0) == binding.FTK_EINVAL
    assert L.ftk_sgd_step_noalloc(None, 0.0, 0.0, 0.0, 0.0) == binding.FTK_EINVAL
    assert L.ftk_rmse(None, C.byref(d)) == binding.FTK_EINVAL
    assert L.ftk_mae(None, C.byref(d)) == binding.FTK_EINVAL
    assert L.ftk_evaluate(None, 1, None, None, 0, C.byref(d), C.byref(d)) == binding.FTK_EINVAL
    assert L.ftk_get_factors(None, None, None) == binding.FTK_EINVAL
    assert L.ftk_set_factors(None, None, None) == binding.FTK_EINVAL
    assert L.ftk_get_samples(None, None) == binding.FTK_EINVAL
    assert L.ftk_set_mode(None, 0) == binding.FTK_EINVAL
    assert L.ftk_set_stream(None, None) == binding.FTK_EINVAL
    assert L.ftk_set_timing(None, 1) == binding.FTK_EINVAL
    assert L.ftk_set_kernel(None, b"auto") == binding.FTK_EINVAL
    assert L.ftk_get_table_rows(None, None, None) == binding.FTK_EINVAL
    L.ftk_destroy(None)
    assert L.ftk_kernel_name(None) is not None


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2204_07104_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "ftk_oracle" not in text, f


def test_step_size_schedule_values():
    """gamma_t = alpha / (1 + beta t^1.5) (Section 5.1): exact where t^1.5 is an integer."""
    import math
    assert binding.ftk_step_size(0.009, 0.1, 0) == 0.009                      # t = 0: alpha itself
    assert math.isclose(binding.ftk_step_size(0.009, 0.1, 4), 0.009 / 1.8, rel_tol=1e-15)    # 4^1.5 = 8
    assert math.isclose(binding.ftk_step_size(2.0, 0.5, 9), 2.0 / 14.5, rel_tol=1e-15)       # 9^1.5 = 27
    assert binding.ftk_step_size(1.0, 0.0, 1000) == 1.0                      # beta = 0: constant
    seq = [binding.ftk_step_size(0.005, 0.05, t) for t in range(50)]
    assert all(a > b > 0.0 for a, b in zip(seq, seq[1:]))                    # strictly decreasing, positive
    assert math.isnan(binding.ftk_step_size(1.0, 1.0, -1))
    assert math.isnan(binding.ftk_step_size(1.0, -1.0, 1))                   # denominator 0


def test_plain_c_program_builds_against_the_header_and_links_the_library(tmp_path):
    """include/ftk.h is C99 (-pedantic -Werror), and a C program linked against libftk.so plus the HIP
    runtime gets the documented behaviour from the calls that need no device."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    hip_dir = os.path.dirname(binding.hip_runtime_path())
    if gcc is None:
        pytest.skip("no gcc")
    lib_dir = os.path.dirname(binding.LIB_PATH)
    exe = str(tmp_path / "abi_smoke")
    subprocess.check_call([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic",
                           "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "abi_smoke.c"), "-o", exe,
                           "-L", lib_dir, "-lftk", "-L", hip_dir, "-lamdhip64",
                           "-Wl,-rpath," + lib_dir, "-Wl,-rpath," + hip_dir])
    done = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert done.returncode == 0, done.stdout + done.stderr
    lines = done.stdout.strip().splitlines()
    assert lines[0] == 'create rc=-1 ctx_is_null=1 error="order 0 outside 1..10"'
    assert lines[1] == "null ctx: sample=-1 step=-1 rmse=-1 kernel=none"
    assert float(lines[2].split("=")[1]) == 0.5 / (1.0 + 0.25 * 8.0)
