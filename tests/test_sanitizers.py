"""Host logic of the library and the C oracle under the address and undefined-behaviour sanitizers.

tests/sanitize/driver.cpp calls what the Python CPU tests call (operators, spaces, sampler, mutation, text form,
interpreter, validator with forced rejections, coverage walks, modules, cost model, search on a synthetic latency,
one oracle operator), built from the library's own host sources with -fsanitize=address,undefined; the part that
needs the compiler and the GPU is replaced by stubs.  Any invalid access, leak of a variant, signed overflow or
misaligned access in that code aborts the driver."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2205_13603_amd", "csrc")


def test_host_logic_and_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "ms_sanitized")
    obj = str(tmp_path / "ms_oracle.o")
    flags = ["-g", "-O1", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
    subprocess.run(["gcc", "-std=c99", "-c"] + flags + ["-o", obj, os.path.join(ROOT, "oracle", "ms_oracle.c")], check=True)
    srcs = [os.path.join(CSRC, f) for f in ("ms_core.cpp", "ms_interp.cpp", "ms_model.cpp", "ms_search.cpp")]
    srcs += [os.path.join(ROOT, "tests", "sanitize", f) for f in ("gpu_stubs.cpp", "driver.cpp")]
    r = subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra"] + flags + ["-I", os.path.join(ROOT, "include"), "-o", exe] + srcs + [obj, "-lm"],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)  # the sanitizer runtime must come first in the driver's own process
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    sys.stdout.write(r.stdout[-2000:])
    assert r.returncode == 0, r.stdout[-6000:]
    assert "sanitized host checks ok" in r.stdout
