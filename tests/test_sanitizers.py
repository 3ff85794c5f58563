"""The CPU-side code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU involved):
the oracle (gcc build) re-runs every one of its pins, and the host code of the HIP library (argument checks,
threshold algorithms, workspace arithmetic; hipcc's host pass) re-runs the host-only boundary tests.
Each runs in a child process with the matching sanitizer runtime preloaded."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(env_extra, preload, tests):
    env = dict(os.environ)
    env.update(env_extra)
    env["LD_PRELOAD"] = preload + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # leak checking needs ptrace, and python itself never frees everything; link order: other preloads may exist
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *tests]
    res = subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-4000:]
    assert " passed" in res.stdout and "runtime error" not in res.stdout and "AddressSanitizer" not in res.stdout
    return res.stdout


def test_oracle_pins_hold_under_asan_and_ubsan():
    libasan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    assert os.path.exists(libasan)
    tests = sorted("tests/" + f for f in os.listdir(os.path.join(ROOT, "tests")) if f.startswith("test_oracle_"))
    assert len(tests) >= 6
    _run({"SF_ORACLE_SANITIZE": "1"}, libasan, tests)


def test_library_host_code_under_asan_and_ubsan():
    from paper_2402_03694_amd import build
    lib = build.build_host_sanitized()
    # test_oracle_per_class.py drives sf_per_class_thresholds, test_calibration.py Algorithm 1 and the
    # target-portion rule, test_abi_host.py the argument checks and exact threshold arithmetic
    _run({"SERVEFLOW_LIB": lib}, build.asan_runtime(),
         ["tests/test_abi_host.py", "tests/test_calibration.py", "tests/test_oracle_per_class.py"])
