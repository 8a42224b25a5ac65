"""CPU-side checks of the C-ABI library: it loads, exports what include/drot.h declares, and its
argument validation answers without a GPU (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2305_18483_amd import binding

    if not os.path.exists(binding.LIB_PATH):
        from paper_2305_18483_amd import build

        build.build()
    return binding.load_library()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "drot.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(drot_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2305_18483_amd import binding

    declared = _declared_functions()
    assert declared, "no declarations found in include/drot.h"
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in drot.h but not exported by libdrot.so"
    assert sorted(binding.EXPORTED_SYMBOLS) == declared


def test_argument_validation_without_a_gpu(lib):
    from paper_2305_18483_amd import binding

    h = ctypes.c_void_p()
    assert lib.drot_create(None, 4, 4) == binding.DROT_ERR_INVALID_ARG
    assert lib.drot_create(ctypes.byref(h), 0, 4) == binding.DROT_ERR_INVALID_ARG
    assert lib.drot_create(ctypes.byref(h), 4, -1) == binding.DROT_ERR_INVALID_ARG
    assert lib.drot_destroy(None) == binding.DROT_ERR_INVALID_ARG
    assert lib.drot_set_option(None, binding.DROT_OPT_CHECK_EVERY, 10) == binding.DROT_ERR_INVALID_ARG
    assert lib.drot_set_gap_tolerance(None, 0.1) == binding.DROT_ERR_INVALID_ARG
    assert lib.drot_get_info(None, None) == binding.DROT_ERR_INVALID_ARG
    assert lib.drot_solve(None, None, None, None, 1, 1, 0.0, 0, None, 1, 0.0, None, None) == binding.DROT_ERR_INVALID_ARG
    for code in (0, 1, -1, -2, -3, -4, 99):
        assert isinstance(binding.strerror(code), str) and binding.strerror(code)


def test_struct_layouts_match_the_header():
    from paper_2305_18483_amd import binding

    # drot_info: int, int, float, float, double x3 ; drot_reg_params: float, float, int, pointer, pointer
    assert ctypes.sizeof(binding.drot_info) == 40
    assert binding.drot_info.objective.offset == 16
    assert ctypes.sizeof(binding.drot_check) == 40 and binding.drot_check.objective.offset == 16
    assert ctypes.sizeof(binding.drot_sweep_timing) == 24 and binding.drot_sweep_timing.c_fraction.offset == 8
    assert ctypes.sizeof(binding.drot_reg_params) == 32
    assert binding.drot_reg_params.row_class.offset == 16
    assert binding.drot_reg_params.weights.offset == 24


def test_input_generators_are_seeded_and_normalised():
    import numpy as np

    import drot_inputs

    a, b = drot_inputs.config(1), drot_inputs.config(1)
    assert np.array_equal(a.C, b.C) and a.C.dtype == np.float32 and a.C.max() == 1.0 and a.C.min() >= 0.0
    assert abs(float(a.p.sum()) - 1.0) < 1e-5 and abs(float(a.q.sum()) - 1.0) < 1e-5
    g = drot_inputs.config(5, size=200)
    assert g.row_class.shape == (200,) and g.num_classes == 10 and (np.diff(g.row_class) >= 0).all()
    r = drot_inputs.random_problem(17, 9, seed=4, reg_kind=2, num_classes=3, sorted_classes=False)
    assert r.C.shape == (17, 9) and r.row_class.max() < 3


def test_bench_refuses_more_than_one_gpu():
    # the benchmark runs on one GPU only: any other count ends at once, before anything touches a device
    import subprocess
    import sys

    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                          stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=120)
    assert proc.returncode == 2
    assert "one GPU" in proc.stderr and proc.stdout.strip() == ""


def test_product_package_does_not_import_the_oracle():
    # the oracle is test infrastructure: nothing under the package may import or name it
    pkg = os.path.join(ROOT, "paper_2305_18483_amd")
    for base, _, files in os.walk(pkg):
        for name in files:
            if name.endswith((".py", ".h", ".hip")):
                text = open(os.path.join(base, name)).read()
                assert "oracle" not in text.lower(), os.path.join(base, name)


def test_kernels_are_built_without_compiler_chosen_fma_contraction():
    # the sweeps promise each other the same bits (screened against unscreened, lean against 8-wave tiles, stored
    # cost against point clouds); that holds only if a product and a sum are fused where the source says fmaf and
    # nowhere else: left to the compiler, fusion depends on which statements happen to share a basic block
    from paper_2305_18483_amd import build
    assert "-ffp-contract=off" in build.HIPCC_FLAGS
    # and packed fp32 instructions stay out of the generated code
    flags = " ".join(build.HIPCC_FLAGS)
    assert "-Xclang -target-feature -Xclang -packed-fp32-ops" in flags


def test_public_header_is_plain_c(tmp_path):
    # the boundary is a C ABI: include/drot.h must compile as C99 on its own, with warnings as errors
    import shutil
    import subprocess

    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler on this machine")
    src = tmp_path / "use_header.c"
    src.write_text('#include "drot.h"\nint main(void) { drot_handle h = 0; drot_info i; (void)h; (void)i; return 0; }\n')
    proc = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                           "-c", str(src), "-o", str(tmp_path / "use_header.o")],
                          stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert proc.returncode == 0, proc.stdout
