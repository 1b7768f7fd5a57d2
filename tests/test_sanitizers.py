"""Sanitizer leg (CPU only): the C oracle and the library's host-side design routines, rebuilt
with gcc/g++ -fsanitize=address,undefined, run their own tests in processes of their own.  The
GPU code is not involved: only plain host sources are instrumented."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _env(extra=None):
    from oracle import build as OB
    env = dict(os.environ)
    runtime = OB.sanitizer_runtime()
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")   # libasan comes first
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=97"      # the interpreter itself is not leak-clean
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:exitcode=98"
    env["OMP_NUM_THREADS"] = "4"
    env.update(extra or {})
    return env


def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    from oracle import build as OB
    lib = OB.build_sanitized()
    cmd = [sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
           os.path.join(ROOT, "tests", "test_oracle_stages.py"), os.path.join(ROOT, "tests", "test_oracle_philox.py"),
           os.path.join(ROOT, "tests", "test_oracle_bucket.py"),
           os.path.join(ROOT, "tests", "test_oracle_quantizer.py")]
    r = subprocess.run(cmd, cwd=ROOT, env=_env({"AGC_ORACLE_LIB": lib}), capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail


def test_host_design_routines_under_address_and_undefined_behaviour_sanitizers():
    from paper_2605_15890_amd import build as HB
    lib = HB.build_host_sanitized()
    r = subprocess.run([sys.executable, os.path.join(ROOT, "tests", "host_routines_driver.py"), lib], cwd=ROOT,
                       env=_env(), capture_output=True, text=True, timeout=600)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "host routines ok" in r.stdout and "runtime error" not in tail, tail
