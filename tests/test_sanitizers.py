"""The CPU side under AddressSanitizer and UndefinedBehaviorSanitizer: the oracle (plain C) runs its
whole pin suite instrumented, and the library's host code (argument checks, planning, launch paths
that reject before any launch) runs the ABI tests instrumented.  Each runs in a child process with
the matching sanitizer runtime preloaded (gcc's for the oracle, clang's for the HIP host code)."""
import glob
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_child(tests, extra_env, runtime):
    env = dict(os.environ)
    env.update(extra_env)
    pre = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = runtime + (":" + pre if pre else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + tests,
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    return r.stdout


def test_oracle_pin_suite_under_sanitizers():
    import oracle
    oracle.build(sanitize=True)
    tests = sorted(glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py")))
    assert len(tests) >= 6
    out = run_child(tests, {"RADAR_ORACLE_SANITIZE": "1"}, oracle.sanitizer_runtime())
    assert " passed" in out


def test_library_host_code_under_sanitizers():
    from paper_2512_14069_amd import build
    build.build_library(force=False, sanitize=True)
    out = run_child([os.path.join(ROOT, "tests", "test_library_abi.py")], {"RADAR_LIB_SANITIZE": "1"},
                    build.sanitizer_runtime())
    assert " passed" in out
