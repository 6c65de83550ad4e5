"""Host-side sanitizer run over the corrupt-input paths: the oracle and the library's CPU sources (model load /
create / fit of both block formats) are compiled with -fsanitize=address,undefined into one program
(tests/sanitize/corrupt_input_main.cpp) that feeds them arbitrary bytes in exactly-sized heap buffers.  A read
or write outside a buffer, or undefined arithmetic, makes the program exit non-zero.  No GPU code is built or
run: decoders must not read outside a block whatever its bytes are, and this is where that is checked for the
CPU side (the GPU side is checked against the oracle's output on the same bytes).
"""
from __future__ import annotations

import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2505_06901_amd", "csrc")


CLANG = "/opt/rocm/llvm/bin/clang++"  # the library's CPU sources use _Float16, which this image's g++ lacks in C++


@pytest.mark.skipif(not os.path.exists(CLANG), reason="needs ROCm's clang++")
def test_corrupt_input_paths_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "corrupt_input")
    sources = [os.path.join(ROOT, "tests", "sanitize", "corrupt_input_main.cpp"),
               os.path.join(ROOT, "oracle", "ecco_oracle.cpp"), os.path.join(ROOT, "oracle", "ecco_paper_block.cpp"),
               os.path.join(CSRC, "ecco_fit.cpp"), os.path.join(CSRC, "ecco_model.cpp"), os.path.join(CSRC, "ecco_pb_model.cpp")]
    # clang links its sanitizer runtimes statically into the program (no runtime library that would have to come
    # first in the load order); OpenMP is left off, so the oracle's group loops run serially
    cmd = [CLANG, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-ffp-contract=off",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-Wno-unknown-pragmas",
           "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
           *sources, "-o", exe, "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-lpthread"]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-4000:]
    env = dict(os.environ)
    # the HIP runtime is linked only because the model sources name its upload calls; nothing here calls them, and
    # what that library allocates when it is loaded is not this code's to free
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-6000:])
    assert run.stdout.count("clean") == 3
