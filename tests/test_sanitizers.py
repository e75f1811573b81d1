"""Host-side sanitizers (no GPU involved).

1. The CPU oracle is rebuilt with AddressSanitizer + UndefinedBehaviorSanitizer and its pins run
   against that build: an out-of-bounds index, a shift past the word or a signed overflow in
   the reference would stop the run.
2. The product library is rebuilt with the same sanitizers on its HOST code (argument
   validation, planning, dispatch: everything that runs before a kernel launch; the device code
   is compiled as usual) and the host-only C-ABI tests run against that build.
Both child runs preload the matching sanitizer runtime into an uninstrumented python; leak
checking is off (the interpreter itself leaks by design), every other finding is fatal.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_child(files, extra_args, preload, tmp_path):
    env = dict(os.environ)
    old = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = preload + (":" + old if old else "")          # the sanitizer runtime has to come first
    env["ASAN_OPTIONS"] = "detect_leaks=0:alloc_dealloc_mismatch=0:detect_odr_violation=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *extra_args,
           *[os.path.join(ROOT, "tests", f) for f in files]]
    res = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    tail = res.stdout[-3000:] + res.stderr[-3000:]
    assert res.returncode == 0, tail
    assert " passed" in res.stdout and "Sanitizer" not in tail and "runtime error" not in tail, tail


def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    so = tmp_path / "liboracle_san.so"
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
                    "-o", str(so), os.path.join(ROOT, "oracle", "pdelta_oracle.c"), "-lm"], check=True)
    libasan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True, check=True).stdout.strip()
    assert os.path.isabs(libasan), "gcc has no shared AddressSanitizer runtime"
    run_child(["test_oracle_formats.py", "test_oracle_pack.py", "test_oracle_linear.py", "test_oracle_group.py"],
              ["--oracle-lib", str(so)], libasan, tmp_path)


def test_host_dispatch_and_validation_under_asan_and_ubsan(tmp_path):
    from paper_2512_19720_amd import build as b
    runtime = b.sanitizer_runtime()
    if not runtime or not os.path.exists(runtime):
        pytest.skip("the ROCm toolchain ships no shared AddressSanitizer runtime")
    so = tmp_path / "libpdelta_san.so"
    obj = tmp_path / "obj"
    b.build_library(jobs=8, lib_path=str(so), obj_dir=str(obj), extra_compile=b.SANITIZE_COMPILE,
                    extra_link=b.SANITIZE_LINK)
    run_child(["test_abi_host.py", "test_zz_no_alloc.py"], ["--pdelta-lib", str(so), "-m", "not gpu"], runtime, tmp_path)
