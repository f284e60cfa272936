"""CPU sanitizer target: the C oracle and the pure-host plan code of the library, built with
gcc/g++ -fsanitize=address,undefined and exercised (brute-force pin of the oracle; plan creation,
splitting, outliers, item walk and argument errors; cost model, retention order, rotary table)
in a subprocess with the sanitizer runtime preloaded.  Any report fails the test."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
       "-O1", "-g", "-shared", "-fPIC"]


def _runtime(name: str) -> str:
    path = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True,
                          check=True).stdout.strip()
    if not os.path.isabs(path) or not os.path.exists(path):
        pytest.skip(f"{name} is not installed")
    return path


def test_oracle_and_host_plan_under_asan_and_ubsan(tmp_path):
    asan = _runtime("libasan.so")
    oracle_so = str(tmp_path / "libpv_oracle_san.so")
    subprocess.run(["gcc", "-std=c11", "-fopenmp", "-Wall"] + SAN
                   + ["-o", oracle_so, os.path.join(ROOT, "oracle", "pv_oracle.c"), "-lm"],
                   check=True, cwd=os.path.join(ROOT, "oracle"))
    # the plan is pure host code; the only entry point it lacks without the GPU part of the library
    # is the destructor, which for a plan that was never uploaded is a plain delete
    stub = tmp_path / "destroy_stub.cpp"
    stub.write_text('#include "pv_plan.h"\nextern "C" void pv_plan_destroy(pv_plan *p) { delete p; }\n')
    plan_so = str(tmp_path / "libpv_plan_san.so")
    csrc = os.path.join(ROOT, "paper_2312_05516_amd", "csrc")
    subprocess.run(["g++", "-std=c++17", "-Wall"] + SAN
                   + ["-I", os.path.join(ROOT, "include"), "-I", csrc, "-o", plan_so,
                      os.path.join(csrc, "pv_plan.cpp"), str(stub)], check=True)
    env = dict(os.environ, LD_PRELOAD=asan, OMP_NUM_THREADS="2",
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:exitcode=23",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([sys.executable, os.path.join(HERE, "sanitizer_driver.py"), oracle_so, plan_so],
                       env=env, capture_output=True, text=True, timeout=600)
    report = r.stdout[-3000:] + r.stderr[-6000:]
    assert r.returncode == 0, report
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, report
    assert "oracle under sanitizers: ok" in r.stdout and "host plan under sanitizers: ok" in r.stdout
