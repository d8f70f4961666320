"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the host-side code: the product's schedulers,
dataflow-graph runtime and tree-generation program (sequential mode; the hand-written fiber switch changes
stacks behind the sanitizer's back and is not run), and the CPU oracle.  Each is a small driver under
tests/sanitize/ compiled with the sources it exercises and run as a program of its own (the sanitizer
runtimes are linked statically, so nothing has to be preloaded)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2305_10611_amd", "csrc")
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan"]


def build_and_run(tmp_path, compiler, std, sources, name, libs):
    if shutil.which(compiler) is None:
        pytest.skip(f"{compiler} is not installed")
    exe = os.path.join(str(tmp_path), name)
    cmd = [compiler, std, *SAN, "-I", os.path.join(ROOT, "include"), "-I", CSRC, *sources, "-o", exe, *libs]
    built = subprocess.run(cmd, capture_output=True, text=True)
    assert built.returncode == 0, built.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    ran = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert ran.returncode == 0 and ran.stdout.strip().endswith(": ok"), (ran.stdout + ran.stderr)[-4000:]


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    src = [os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp")]
    src += [os.path.join(CSRC, f) for f in ("scheduler.cpp", "dfg_runtime.cpp", "tdc_runtime.cpp", "fiber.cpp")]
    build_and_run(tmp_path, "g++", "-std=c++17", src, "host_driver", ["-lpthread"])


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    src = [os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), os.path.join(ROOT, "oracle", "acrobat_oracle.c")]
    build_and_run(tmp_path, "gcc", "-std=c11", src, "oracle_driver", ["-lm", "-lpthread"])
