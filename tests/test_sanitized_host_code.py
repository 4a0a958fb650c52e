"""The host-side code under AddressSanitizer and UndefinedBehaviorSanitizer: the C oracle, and the library's
argument validation, chunk-size selector (paper section 4.4), graph registrar / first-fit planner / chunk search
(sections 4.3 - 4.5) and VMM object are rebuilt with both sanitizers, and the CPU tests that exercise them run
again, in a child process, against those builds.  Device code is not involved (kernel launchers are replaced by
stand-ins; no test here launches anything)."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2601_06562_amd", "csrc")
CLANG = "/opt/rocm/llvm/bin/clang"
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SAN = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
       "-shared-libsan", "-fPIC", "-shared"]
TESTS = ["test_oracle_pins.py", "test_planner_oracle_pins.py", "test_planner_trace_pin.py", "test_host_api.py",
         "test_graph_planner.py"]


def asan_runtime():
    found = glob.glob("/opt/rocm/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    return found[0] if found else None


@pytest.mark.skipif(not (os.path.exists(CLANG) and asan_runtime()), reason="no clang sanitizer runtime in this image")
def test_cpu_tests_pass_against_sanitizer_builds(tmp_path):
    oracle_lib = str(tmp_path / "libmosaic_oracle_san.so")
    host_lib = str(tmp_path / "libmosaic_host_san.so")
    subprocess.run([CLANG, *SAN, "-fopenmp", "-std=c11", "-o", oracle_lib, os.path.join(ROOT, "oracle", "mosaic_oracle.c"),
                    "-lm"], check=True, stderr=subprocess.DEVNULL)
    sources = [os.path.join(CSRC, f) for f in ("mosaic_api.hip", "mosaic_vmm.hip", "mosaic_plan.cpp", "mosaic_graph.cpp")]
    sources.append(os.path.join(ROOT, "tests", "sanitizer_launch_stubs.cpp"))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-std=c++17", *SAN, "-Wno-unused-command-line-argument",
                    "-Wno-option-ignored", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-o", host_lib, *sources],
                   check=True, stderr=subprocess.DEVNULL)
    env = dict(os.environ)
    preload = [asan_runtime()] + [p for p in env.get("LD_PRELOAD", "").split(":") if p]
    env.update(LD_PRELOAD=":".join(preload), MOSAIC_TEST_LIBRARY=host_lib, MOSAIC_TEST_ORACLE_LIBRARY=oracle_lib,
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="4")
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu",
           *[os.path.join(ROOT, "tests", t) for t in TESTS]]
    res = subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)
    tail = res.stdout[-4000:]
    assert "AddressSanitizer" not in res.stdout and "runtime error:" not in res.stdout, tail
    assert res.returncode == 0, tail
    assert " passed" in res.stdout and "failed" not in res.stdout.splitlines()[-1], tail
