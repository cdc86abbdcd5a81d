"""The CPU side under sanitizers (no GPU): the oracle's pins against a build of the oracle with AddressSanitizer and
UndefinedBehaviorSanitizer, and the host-side argument checking of the HIP library against a build of it whose host code
is compiled with the same two (device code cannot be sanitized here and is not run by these tests).  Each runs in a
process of its own with the sanitizer runtime preloaded."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _env(preload, **extra):
    env = dict(os.environ)
    prior = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = preload + (":" + prior if prior else "")         # the sanitizer runtime has to come first
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"        # the interpreter itself leaks by design
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env.update(extra)
    return env


def test_oracle_pins_pass_under_asan_and_ubsan():
    rt = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(rt) or not os.path.exists(rt):
        pytest.skip("gcc's libasan.so is not installed")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       cwd=ROOT, env=_env(rt, EQAT_ORACLE_SANITIZE="1", OMP_NUM_THREADS="4"), capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail


def test_host_side_of_the_library_passes_its_abi_and_work_plan_tests_under_asan_and_ubsan(tmp_path):
    import glob
    rts = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not rts:
        pytest.skip("the ROCm compiler's AddressSanitizer runtime is not installed")
    lib = tmp_path / "libeqat_hostsan.so"
    flags = "-Xarch_host -fsanitize=address -Xarch_host -fsanitize=undefined -Xarch_host -fno-omit-frame-pointer -g"
    b = subprocess.run([sys.executable, "-m", "paper_2407_11062_amd.build"], cwd=ROOT, capture_output=True, text=True, timeout=1500,
                       env=dict(os.environ, EQAT_EXTRA_FLAGS=flags, EQAT_EXTRA_LINK_FLAGS="-fsanitize=address -fsanitize=undefined -shared-libsan",
                                EQAT_OBJ_DIR=str(tmp_path / "obj"), EQAT_LIB_OUT=str(lib), EQAT_PEAKS_LIB_OUT=str(tmp_path / "libpeaks.so")))
    assert b.returncode == 0, (b.stdout + b.stderr)[-3000:]
    # (all of them but the one that links a plain gcc program against the library: that program has no sanitizer runtime)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-k", "not plain_c",
                        os.path.join(ROOT, "tests", "test_host_abi.py"), os.path.join(ROOT, "tests", "test_work_plan.py")],
                       cwd=ROOT, env=_env(rts[0], EQAT_LIB=str(lib)), capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
