"""Sanitizer builds of the host code (no GPU): the oracle under AddressSanitizer and
UndefinedBehaviorSanitizer, the oracle's pins through a UBSan build, and the argument checks of
libdass through a build whose host code carries both sanitizers."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TESTS = os.path.join(ROOT, "tests")
ORACLE_C = os.path.join(ROOT, "oracle", "dass_oracle.c")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
# a sanitizer report must fail the run whatever the defaults are
SAN_ENV = dict(os.environ, ASAN_OPTIONS="abort_on_error=0:exitcode=97:detect_leaks=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="halt_on_error=1:exitcode=98:print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-2000:]}\n{r.stderr[-4000:]}"
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    return r.stdout


def test_oracle_under_asan_and_ubsan(tmp_path):
    """Every oracle function on ragged inputs in exact-size heap blocks: no report, and the same
    results as the ordinary build."""
    driver = os.path.join(TESTS, "oracle_sanitizer_driver.c")
    common = ["gcc", "-std=gnu11", "-ffp-contract=off", "-fopenmp", driver, ORACLE_C, "-lm"]
    plain, checked = str(tmp_path / "plain"), str(tmp_path / "checked")
    _run(common + ["-O2", "-o", plain])
    _run(common + ["-O1", "-g", "-static-libasan", "-o", checked] + SAN)
    want = _run([plain])
    got = _run([checked], env=SAN_ENV)
    assert got == want and want.rstrip().endswith("all ok") and want.count("\n") > 200


def test_oracle_pins_through_a_ubsan_build(tmp_path):
    """The pins of tests/test_oracle_*.py run again with the oracle compiled with
    -fsanitize=undefined (a shared object with that runtime loads into an ordinary interpreter)."""
    lib = str(tmp_path / "libdass_oracle_ubsan.so")
    _run(["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-std=gnu11", "-ffp-contract=off",
          "-fsanitize=undefined", "-fno-sanitize-recover=all", "-o", lib, ORACLE_C, "-lm"])
    pins = sorted(f for f in os.listdir(TESTS) if f.startswith("test_oracle_") and f.endswith(".py"))
    assert len(pins) >= 4
    out = _run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + [os.path.join(TESTS, f) for f in pins],
               env=dict(SAN_ENV, DASS_ORACLE_LIB=lib), cwd=ROOT)
    assert " passed" in out and "failed" not in out


def test_library_argument_checks_under_host_sanitizers(tmp_path):
    """libdass built with ASan + UBSan on the host side; a driver makes every rejected call of
    include/dass.h's entry points.  Expected status names are listed here."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    clangxx = "/opt/rocm/lib/llvm/bin/clang++"
    if not (os.path.exists(hipcc) and os.path.exists(clangxx)):
        pytest.skip("no ROCm toolchain")
    sys.path.insert(0, ROOT)
    from paper_2405_01943_amd import build as lib_build

    host_san = []
    for flag in SAN:
        host_san += ["-Xarch_host", flag]
    flags = [f for f in lib_build.HIPCC_FLAGS if f != "-O3"] + ["-O1"] + host_san
    procs = []
    for src in lib_build.sources():
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        procs.append((obj, subprocess.Popen([hipcc] + flags + ["-c", src, "-o", obj], stdout=subprocess.PIPE,
                                            stderr=subprocess.PIPE, text=True)))
    objs = []
    for obj, p in procs:
        _, err = p.communicate(timeout=900)
        assert p.returncode == 0, err[-3000:]
        objs.append(obj)
    exe = str(tmp_path / "abi_driver")
    _run([clangxx, "-std=c++17", "-O1", "-g"] + SAN + ["-o", exe, os.path.join(TESTS, "abi_sanitizer_driver.cpp")] + objs +
         ["-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"])
    out = _run([exe], env=SAN_ENV)
    got = dict(line.split(" ", 1) for line in out.strip().splitlines())
    assert "MISSING-ERROR-TEXT" not in out and out.rstrip().endswith("all ok")
    want = {
        "nm_null_W": "DASS_ERR_NULL", "nm_null_norms": "DASS_ERR_NULL", "nm_dtype": "DASS_ERR_DTYPE",
        "nm_rows0": "DASS_ERR_SHAPE", "nm_ld": "DASS_ERR_SHAPE", "nm_cols8": "DASS_ERR_SHAPE",
        "nm_ragged_groups": "DASS_ERR_SHAPE", "nm_m3": "DASS_ERR_ARG", "nm_keep_all": "DASS_ERR_ARG",
        "nm_alpha_nan": "DASS_ERR_ARG", "nm_alpha_neg": "DASS_ERR_ARG", "nm_axis": "DASS_ERR_ARG",
        "nm_align": "DASS_ERR_ALIGN", "nm_ld_align": "DASS_ERR_ALIGN", "nm_no_ws": "DASS_ERR_WORKSPACE",
        "nm_small_ws": "DASS_ERR_WORKSPACE", "nm_huge": "DASS_ERR_SHAPE",
        "batched_empty": "DASS_OK", "batched_null_task1": "DASS_ERR_NULL", "batched_shape_task2": "DASS_ERR_SHAPE",
        "batched_null_array": "DASS_ERR_NULL", "batched_negative": "DASS_ERR_NULL",
        "un_neg": "DASS_ERR_ARG", "un_too_many": "DASS_ERR_ARG", "un_no_ws": "DASS_ERR_WORKSPACE",
        "un_null": "DASS_ERR_NULL", "un_cols": "DASS_ERR_SHAPE", "un_static_limit": "DASS_ERR_WORKSPACE",
        "calib_null": "DASS_ERR_NULL", "calib_null_sumsq": "DASS_ERR_NULL", "calib_dtype": "DASS_ERR_DTYPE",
        "calib_act": "DASS_ERR_DTYPE", "calib_T0": "DASS_ERR_SHAPE", "calib_d8": "DASS_ERR_SHAPE",
        "calib_ldx": "DASS_ERR_SHAPE", "calib_align": "DASS_ERR_ALIGN", "calib_ldw_align": "DASS_ERR_ALIGN",
        "calib_too_many_tiles": "DASS_ERR_SHAPE", "calib_too_many_tiles_f32": "DASS_ERR_SHAPE",
        "calib_too_many_tiles_ragged_d": "DASS_ERR_SHAPE",
        "in_null": "DASS_ERR_NULL", "in_dtype": "DASS_ERR_DTYPE", "in_T0": "DASS_ERR_SHAPE", "in_d": "DASS_ERR_SHAPE",
        "in_align": "DASS_ERR_ALIGN", "in_ws": "DASS_ERR_WORKSPACE",
        "fwd_null": "DASS_ERR_NULL", "fwd_out_null": "DASS_ERR_NULL", "fwd_dtype": "DASS_ERR_DTYPE",
        "fwd_T0": "DASS_ERR_SHAPE", "fwd_d64": "DASS_ERR_SHAPE", "fwd_align": "DASS_ERR_ALIGN",
        "fwd_ldo": "DASS_ERR_ALIGN", "fwd_ws": "DASS_ERR_WORKSPACE",
        "cmp_null": "DASS_ERR_NULL", "cmp_meta_null": "DASS_ERR_NULL", "cmp_dtype": "DASS_ERR_DTYPE",
        "cmp_axis": "DASS_ERR_ARG", "cmp_cols": "DASS_ERR_SHAPE", "cmp_rows4": "DASS_ERR_SHAPE",
        "cmp_ldv": "DASS_ERR_SHAPE", "cmp_align": "DASS_ERR_ALIGN", "cmp_surplus_align": "DASS_ERR_ALIGN",
        "cmp_overlap": "DASS_ERR_ARG",
        "spd_null": "DASS_ERR_NULL", "spd_dtype": "DASS_ERR_DTYPE", "spd_T0": "DASS_ERR_SHAPE",
        "spd_d8": "DASS_ERR_SHAPE", "spd_ldm": "DASS_ERR_SHAPE", "spd_ldm_align": "DASS_ERR_ALIGN",
        "spd_ldo": "DASS_ERR_ALIGN", "unknown_status": "DASS_ERR_UNKNOWN",
    }
    for label, status in want.items():
        assert got.get(label) == status, f"{label}: got {got.get(label)}, want {status}"
    assert "task 1" in got["batched_text"]
    assert int(got["nm_ws_bytes"]) >= 4 * 11008 and int(got["fwd_ws_bytes"]) == 256 * 192 * 2
    shutil.rmtree(tmp_path, ignore_errors=True)
