"""The oracle under the compiler's sanitizers (CPU only).

Every parity claim rests on ``oracle/rc_oracle.c``; a read past an array or a signed overflow in it would be
a silent error in the checker.  Two builds, both on the host:
  * ``oracle/sanitize_driver.c`` + the oracle as one program with AddressSanitizer and
    UndefinedBehaviorSanitizer (no Python in the process): calls every oracle function on small random problems
    held in exact-size heap buffers.  It must end cleanly, and its checksum must equal the plain build's.
  * the oracle as a shared library with UndefinedBehaviorSanitizer (errors are fatal): the whole pin suite runs
    against it in a child process and must pass.
"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE = os.path.join(ROOT, "oracle")


def _run(cmd, **kw):
    return subprocess.run(cmd, capture_output=True, text=True, timeout=900, **kw)


def test_every_oracle_function_is_clean_under_asan_and_ubsan(tmp_path):
    src = [os.path.join(ORACLE, "sanitize_driver.c"), os.path.join(ORACLE, "rc_oracle.c")]
    plain, san = str(tmp_path / "plain"), str(tmp_path / "san")
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-o", plain] + src + ["-lm"])
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-o", san] + src + ["-lm"])
    env = dict(os.environ, OMP_NUM_THREADS="2", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    a, b = _run([plain], env=env), _run([san], env=env)
    assert a.returncode == 0, a.stdout + a.stderr
    assert b.returncode == 0, b.stdout[-2000:] + b.stderr[-4000:]
    assert a.stdout.startswith("checksum ") and a.stdout == b.stdout


def test_pin_suite_passes_on_a_ubsan_build_of_the_oracle(tmp_path):
    lib = str(tmp_path / "librc_oracle_ubsan.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-fsanitize=undefined",
                           "-fno-sanitize-recover=all", "-o", lib, os.path.join(ORACLE, "rc_oracle.c"), "-lm"])
    env = dict(os.environ, RC_ORACLE_LIB=lib, UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = _run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
              "-p", "no:cacheprovider"], cwd=ROOT, env=env)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
