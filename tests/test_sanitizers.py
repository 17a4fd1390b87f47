"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU-side code, run on the CPU only:
the oracle (plain C) against its pins, and the library's host-side serving functions (csrc/sched.hip
built with -DREC_HOST_ONLY by a plain g++, no HIP) against the oracle.  The instrumented libraries
are loaded into a child Python with the sanitizer runtime preloaded; any report aborts the child."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]


def _runtime():
    p = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(p) or not os.path.exists(p):
        pytest.skip("no libasan for gcc in this environment")
    return os.path.realpath(p)


def _run_under_sanitizers(tests, extra_env):
    env = dict(os.environ)
    env.update(extra_env)
    preload = [_runtime()] + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else [])
    env["LD_PRELOAD"] = ":".join(preload)
    # the interpreter itself is not instrumented: no leak check at exit, no complaint about link order
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + tests, cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, (r.stdout[-3000:] + "\n" + r.stderr[-3000:])
    assert "passed" in r.stdout


def test_oracle_under_asan_and_ubsan(tmp_path):
    lib = str(tmp_path / "librec_oracle_san.so")
    subprocess.check_call(["gcc"] + SAN + ["-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", lib,
                                            os.path.join(ROOT, "oracle", "rec_oracle.c"), "-lm"])
    _run_under_sanitizers(["tests/test_oracle_pins.py", "tests/test_oracle_sched_pins.py"], {"REC_ORACLE_LIB": lib})


def test_host_serving_code_under_asan_and_ubsan(tmp_path):
    lib = str(tmp_path / "librec_sched_san.so")
    subprocess.check_call(["g++", "-x", "c++", "-std=c++17"] + SAN + ["-DREC_HOST_ONLY", "-I" + os.path.join(ROOT, "include"),
                                                                      "-fPIC", "-shared", "-pthread", "-Wall", "-o", lib,
                                                                      os.path.join(ROOT, "paper_2001_02772_amd", "csrc", "sched.hip")])
    _run_under_sanitizers(["tests/test_sched_host.py"], {"REC_LIB_PATH": lib})
