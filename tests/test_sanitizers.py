"""Host-side sanitizer passes (CPU only, nothing here touches a GPU).

  * the oracle's C source built with AddressSanitizer + UndefinedBehaviorSanitizer and the whole CPU test-suite
    run on that build: an out-of-bounds index, a signed overflow or a misaligned access anywhere in the oracle
    ends the run;
  * the C-ABI's host side (argument checks, size functions, metadata converters' checks: csrc/api.hip) built with
    the same sanitizers for the host pass only, and the ABI host tests run on it.

Both run in a child process with the sanitizer's runtime preloaded (an instrumented shared library needs the
runtime to be in the process before it).
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"]


def _preload(runtime, env):
    env = dict(env)
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # the interpreter itself is not leak-clean; everything else stays fatal
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=0:exitcode=97"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:exitcode=98"
    return env


def _run(cmd, env, timeout):
    res = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=timeout)
    tail = (res.stdout[-3000:] + "\n" + res.stderr[-3000:])
    assert "ERROR: AddressSanitizer" not in res.stdout + res.stderr, tail
    assert "runtime error:" not in res.stdout + res.stderr, tail
    assert res.returncode == 0, tail
    return res


def test_cpu_suite_on_the_instrumented_oracle():
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("gcc has no AddressSanitizer runtime here")
    env = _preload(runtime, os.environ)
    env["DFSS_ORACLE_EXTRA_CFLAGS"] = " ".join(SAN + ["-g", "-fno-omit-frame-pointer"])
    lib = os.path.join(ROOT, "oracle", "liboracle_instrumented.so")
    if os.path.exists(lib):
        os.remove(lib)
    res = _run([sys.executable, "-m", "pytest", "tests", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                "--ignore", os.path.join("tests", "test_sanitizers.py")], env, timeout=1500)
    assert os.path.exists(lib), "the run did not build (so did not use) the instrumented oracle"
    assert " passed" in res.stdout


def test_abi_host_checks_on_the_instrumented_library():
    from paper_2203_00091_amd import build as b
    hipcc = b._hipcc()
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc here")
    clang_dir = subprocess.run([hipcc, "-print-resource-dir"], capture_output=True, text=True).stdout.strip()
    runtime = os.path.join(clang_dir, "lib", "linux", "libclang_rt.asan-x86_64.so")
    if not os.path.exists(runtime):
        pytest.skip("hipcc's clang has no AddressSanitizer runtime here")
    b.build(incremental=True)          # the other objects are the plain ones
    host_san = [x for f in SAN for x in ("-Xarch_host", f)]
    obj = os.path.join(b.OBJ_DIR, "api_host_instrumented.o")
    lib = os.path.join(b.OBJ_DIR, "libdfss_host_instrumented.so")
    subprocess.run([hipcc, *b.HIPCC_FLAGS, *host_san, "-g", "-c", os.path.join(b.CSRC, "api.hip"), "-o", obj],
                   check=True, capture_output=True)
    others = [os.path.join(b.OBJ_DIR, os.path.basename(s)[:-4] + ".o") for s in b.sources()
              if os.path.basename(s) != "api.hip"]
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *host_san, "-shared-libsan", "-o", lib, obj,
                    *others], check=True, capture_output=True)
    code = ("import sys, pytest, paper_2203_00091_amd.binding as b; b._LIB_PATH = %r; "
            "sys.exit(pytest.main(['-x', '-q', '-p', 'no:cacheprovider', 'tests/test_abi_host.py']))" % lib)
    try:
        res = _run([sys.executable, "-c", code], _preload(runtime, os.environ), timeout=900)
    finally:
        os.remove(lib)
        os.remove(obj)
    assert " passed" in res.stdout
