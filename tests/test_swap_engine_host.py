"""The swap engine's host logic under the address and undefined-behaviour sanitizers, without a GPU: the engine and
planner sources are compiled with g++ against a stand-in for the HIP runtime (tests/host/hip_stub) together with
tests/host/swap_engine_host_test.cpp, which drives the C ABI through its states, error paths and arena rules."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOST = os.path.join(ROOT, "tests", "host")
CSRC = os.path.join(ROOT, "paper_1812_07816_amd", "csrc")


def test_swap_engine_host_logic_under_sanitizers(tmp_path):
    exe = str(tmp_path / "swap_engine_host_test")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
           "-Wall", "-Wextra", "-Wno-unused-parameter", "-I", os.path.join(HOST, "hip_stub"),
           os.path.join(HOST, "swap_engine_host_test.cpp"), os.path.join(CSRC, "swap_engine.cpp"), os.path.join(CSRC, "swap_planner.cpp"),
           "-o", exe]
    b = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert b.returncode == 0, b.stdout
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", LD_PRELOAD="")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
    assert r.returncode == 0 and "swap engine host checks passed" in r.stdout, r.stdout
