"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only): the library's planner and routing
functions on random and invalid inputs, the oracle's C code on a tiny batch.  Builds tests/native/sanitize_host.cpp
with g++ against the host sources (no HIP) and runs it."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_planner_routing_and_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_host")
    csrc = os.path.join(ROOT, "paper_2603_13358_amd", "csrc")
    obj = str(tmp_path / "oracle.o")
    flags = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
    subprocess.check_call(["gcc", "-c", "-fopenmp"] + flags + [os.path.join(ROOT, "oracle", "ppd_oracle.c"), "-o", obj])
    subprocess.check_call(["g++", "-std=c++17", "-fopenmp"] + flags +
                          [os.path.join(ROOT, "tests", "native", "sanitize_host.cpp"), os.path.join(csrc, "ppd_plan.cpp"),
                           os.path.join(csrc, "ppd_route.cpp"), obj, "-lm", "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", OMP_NUM_THREADS="2")
    env.pop("LD_PRELOAD", None)
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout[-3000:]
    assert "planner ok" in res.stdout and "routing ok" in res.stdout and "oracle ok" in res.stdout
