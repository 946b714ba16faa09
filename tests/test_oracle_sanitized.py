"""The oracle's own tests once more, with the oracle built under AddressSanitizer and
UndefinedBehaviorSanitizer: an out-of-bounds index, a use after free or signed overflow in the
reference that every GPU result is compared with would otherwise go unnoticed (there is no GPU-side
sanitizer on this machine, so the CPU side is the net under the gathered indices)."""
import os
import subprocess
import sys

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_tests_pass_under_asan_and_ubsan(tmp_path):
    lib = oracle.build_sanitized(str(tmp_path))
    libasan = subprocess.check_output(["g++", "-print-file-name=libasan.so"], text=True).strip()
    assert os.path.isabs(libasan) and os.path.exists(libasan), libasan
    env = dict(os.environ)
    env["LSH_ORACLE_LIB"] = lib
    env["LD_PRELOAD"] = libasan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # (the interpreter itself is not instrumented and never frees everything: no leak report)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    tests = [os.path.join(ROOT, "tests", f) for f in sorted(os.listdir(os.path.join(ROOT, "tests")))
             if f.startswith("test_oracle_") and f != "test_oracle_sanitized.py"]
    assert len(tests) >= 4
    # the child proves that it really runs the instrumented library
    probe = ("import oracle, ctypes; l = oracle._L(); "
             "assert 'asan' in l._name, l._name; "
             "ctypes.CDLL(None).__asan_init; print('instrumented')")
    out = subprocess.run([sys.executable, "-c", probe], env=env, cwd=ROOT, capture_output=True, text=True)
    assert out.returncode == 0 and "instrumented" in out.stdout, out.stderr[-2000:]
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + tests,
                         env=env, cwd=ROOT, capture_output=True, text=True)
    assert run.returncode == 0, (run.stdout[-3000:], run.stderr[-3000:])
    assert " passed" in run.stdout
