"""CPU sanitizer build of the pointer-heavy host code: the oracle's C file and the planner's host-only
translation unit are compiled with -fsanitize=address,undefined (host compiler, no device code) and the
oracle's pins and the planner's tests (paper fixture, scenarios, random traces against the structural
oracle) run again on those builds.  Any report of the sanitizers aborts the run."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def test_oracle_and_planner_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    oracle_so, planner_so = str(tmp_path / "oracle_san.so"), str(tmp_path / "planner_san.so")
    subprocess.run(["gcc", *SAN, "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", "-o", oracle_so,
                    os.path.join(ROOT, "oracle", "alora_oracle.c")], check=True)
    subprocess.run(["g++", "-x", "c++", "-std=c++17", *SAN, "-shared", "-fPIC", "-I", os.path.join(ROOT, "include"),
                    "-o", planner_so, os.path.join(ROOT, "paper_2512_17910_amd", "csrc", "alora_planner.hip")], check=True)
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()
    env = dict(os.environ)
    # the sanitizer's runtime first, whatever was preloaded already behind it
    env["LD_PRELOAD"] = ":".join(p for p in (asan, env.get("LD_PRELOAD", "")) if p)
    # the interpreter itself is not instrumented: no leak report for its own allocations at exit
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([sys.executable, os.path.join(ROOT, "tests", "sanitized_runner.py"), oracle_so, planner_so],
                       env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout[-3000:] + "\n" + r.stderr[-3000:])
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
