"""Sanitizer leg (CPU only; GPU code is never run under a sanitizer here).

1. The oracle, built with gcc's AddressSanitizer and UndefinedBehaviorSanitizer, runs all of its
   pins (``tests/test_oracle_*.py``) in a child process; a planted heap overflow must be caught,
   which shows that the instrumented build is the one that ran.
2. The host side of ``libaht.so``, built by hipcc with the same two sanitizers on the host pass
   only (``-Xarch_host``; the device code is compiled as always and not executed), runs the
   argument-checking paths of ``tests/test_abi.py``.

Commands (what the tests below run):
  gcc -O1 -g -std=c11 -fopenmp -ffp-contract=off -fno-fast-math -fPIC -shared \
      -fsanitize=address,undefined -fno-sanitize-recover=undefined -fno-omit-frame-pointer \
      -o $TMP/liboracle_san.so oracle/pulsed_update_oracle.c -lm
  AHT_ORACLE_LIB=$TMP/liboracle_san.so LD_PRELOAD=$(gcc -print-file-name=libasan.so) \
      ASAN_OPTIONS=detect_leaks=0 python -m pytest tests -m "not gpu" -k "oracle and not mutants and not sanitizer"
  python -m paper_2104_02184_amd.build  with  -Xarch_host -fsanitize=address -Xarch_host -fsanitize=undefined
      -shared-libsan  ->  $TMP/libaht_san.so
  AHT_LIB=$TMP/libaht_san.so LD_PRELOAD=<clang's libclang_rt.asan-x86_64.so> ASAN_OPTIONS=detect_leaks=0 \
      python -m pytest tests/test_abi.py
(leak detection is off: the interpreter itself is not instrumented and never frees much of what it allocates)
"""
import glob
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "pulsed_update_oracle.c")
GCC_SAN = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]


def _preload(runtime):
    cur = os.environ.get("LD_PRELOAD", "")
    return runtime + (":" + cur if cur else "")


def _pytest(args, env):
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + args
    return subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)


def _gcc_asan_runtime():
    if not shutil.which("gcc"):
        pytest.skip("gcc is not installed")
    path = subprocess.run(["gcc", "-print-file-name=libasan.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    if not os.path.isabs(path) or not os.path.exists(path):
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    return path


def test_oracle_pins_are_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    runtime = _gcc_asan_runtime()
    so = str(tmp_path / "liboracle_san.so")
    subprocess.run(GCC_SAN + ["-o", so, SRC, "-lm"], check=True)
    env = dict(os.environ, AHT_ORACLE_LIB=so, LD_PRELOAD=_preload(runtime), ASAN_OPTIONS="detect_leaks=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    r = _pytest([os.path.join(ROOT, "tests"), "-k", "oracle and not mutants and not sanitizer"], env)
    assert r.returncode == 0, r.stdout[-3000:]
    assert "passed" in r.stdout and "ERROR: AddressSanitizer" not in r.stdout and "runtime error:" not in r.stdout

    # the instrumentation is live: a lookup buffer one sample too short must be reported
    text = open(SRC).read()
    a = "uint64_t *xwT = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)C * (size_t)(B > 0 ? B : 1));"
    assert text.count(a) == 1
    bad_c, bad_so = str(tmp_path / "overflow.c"), str(tmp_path / "liboracle_overflow.so")
    with open(bad_c, "w") as f:
        f.write(text.replace(a, a.replace("(B > 0 ? B : 1)", "(B > 1 ? B - 1 : 1)")))
    subprocess.run(GCC_SAN + ["-o", bad_so, bad_c, "-lm"], check=True)
    # (-s: the report goes to the child's stderr, which pytest would otherwise hold back and lose)
    r = _pytest(["-s", os.path.join(ROOT, "tests", "test_oracle_device.py")], dict(env, AHT_ORACLE_LIB=bad_so))
    assert r.returncode != 0 and "heap-buffer-overflow" in r.stdout, r.stdout[-2000:]


def test_library_argument_paths_are_clean_under_host_sanitizers(tmp_path):
    from paper_2104_02184_amd import build as hip_build
    try:
        hip_build.hipcc()
    except RuntimeError:
        pytest.skip("hipcc is not installed")
    found = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not found:
        pytest.skip("clang's AddressSanitizer runtime is not installed")
    so = str(tmp_path / "libaht_san.so")
    hip_build.build(force=True, extra=hip_build.SANITIZE_HOST + ["-shared-libsan"], out=so)
    env = dict(os.environ, AHT_LIB=so, LD_PRELOAD=_preload(found[0]), ASAN_OPTIONS="detect_leaks=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    r = _pytest([os.path.join(ROOT, "tests", "test_abi.py")], env)
    assert r.returncode == 0, r.stdout[-3000:]
    assert "passed" in r.stdout and "ERROR: AddressSanitizer" not in r.stdout and "runtime error:" not in r.stdout
