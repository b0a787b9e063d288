"""AddressSanitizer + UndefinedBehaviorSanitizer builds, on the CPU, of the code that walks
caller-supplied tables on the host: the C oracle (all four files) and the host side of the
library (argument checks, workspace sizing, the table validators).  Each build runs a set of the
existing checks in a child process with the sanitizer runtime preloaded; any report fails."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_child(code: str, runtime: str, extra_env=None):
    env = dict(os.environ)
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["PYTHONPATH"] = ROOT + os.pathsep + os.path.join(ROOT, "tests")
    env.update(extra_env or {})
    res = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=900, cwd=ROOT)
    report = res.stdout[-3000:] + res.stderr[-6000:]
    assert res.returncode == 0, report
    assert "AddressSanitizer" not in res.stderr and "runtime error:" not in res.stderr, report
    return res.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    srcs = sorted(glob.glob(os.path.join(ROOT, "oracle", "optgqa_oracle*.c")))
    assert len(srcs) == 4
    lib = str(tmp_path / "liboracle_asan.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                           "-fno-omit-frame-pointer", "-o", lib, *srcs, "-lm"])
    code = f"""
import oracle as O, pins, pins_e4m3, pins_window, pins_prompt
lib = O.load({lib!r})
n = 0
for mod in (pins, pins_e4m3, pins_window, pins_prompt):
    for check in mod.ALL_CHECKS:
        check(lib)
        n += 1
print("checks run:", n)
"""
    out = run_child(code, runtime, {"OMP_NUM_THREADS": "4"})
    assert "checks run:" in out


def test_library_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """hipcc builds the library with the sanitizers on the HOST pass only (device code unchanged);
    the child process then drives every host-side path that needs no GPU."""
    from paper_2505_02351_amd import build
    rt = sorted(glob.glob("/opt/rocm/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    if not rt:
        pytest.skip("clang's AddressSanitizer runtime is not installed")
    lib = str(tmp_path / "liboptgqa_asan.so")
    cmd = ["hipcc", *build.HIPCC_FLAGS, "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-shared-libsan",
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(build.PKG, "csrc"), build.SRC, "-o", lib]
    res = subprocess.run(cmd, capture_output=True, text=True, cwd=str(tmp_path))
    assert res.returncode == 0, res.stderr[-4000:]
    code = f"""
import ctypes, numpy as np
import paper_2505_02351_amd as G
G.load_library({lib!r})
import test_abi_host as T
T.test_exports_every_declared_symbol(G)
T.test_status_strings(G)
T.test_argument_errors_before_any_launch(G)
T.test_more_entry_points_reject_bad_arguments_before_any_launch(G)
T.test_workspace_query(G)
T.test_validate_tables_host(G)
T.test_static_scratch_entry_point_refuses_what_does_not_fit(G)
T.test_non_finite_scale_is_refused(G)
T.test_shared_prefix_host_checks(G)
T.test_per_head_scale_entry_points_reject_missing_arrays(G)
print("host paths ok")
"""
    out = run_child(code, rt[-1])
    assert "host paths ok" in out
