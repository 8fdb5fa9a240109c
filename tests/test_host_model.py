"""Builds tests/host_model_main.cpp -- the library's HIP-free sources (configuration checks, planner, the tile
arithmetic the kernels share with it) plus the C oracle -- with the host sanitizers and runs it: a host model of
the kernels' key-range walk (every DMA source row in bounds, every visible key fetched exactly once, for plain and
sink + sliding-window steps, fused append or not), a sweep of the planner, and the oracle on tiny inputs."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_model_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "host_model")
    csrc = os.path.join(ROOT, "paper_2605_12471_amd", "csrc")
    obj = str(tmp_path / "oracle.o")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]
    subprocess.run(["gcc", "-O1", *san, "-c", os.path.join(ROOT, "oracle", "kvfold_oracle.c"), "-o", obj], check=True)
    subprocess.run(["g++", "-std=c++17", "-O2", *san, os.path.join(ROOT, "tests", "host_model_main.cpp"),
                    os.path.join(csrc, "kvfold_plan.cpp"), obj, "-lm", "-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)   # the sanitizer runtime has to come first in the new process
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    assert "ok:" in r.stdout
