"""The CPU oracle under sanitizers (gcc, host only): its entry points walked over edge shapes in an AddressSanitizer +
UBSan build, and its pins run once against a UBSan build of the library."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_edge_shapes_under_asan_and_ubsan_match_the_regular_build():
    from oracle.build import build_sanitized
    _, san, plain = build_sanitized()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1", OMP_NUM_THREADS="2")
    a = subprocess.run([san], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=env, timeout=300)
    assert a.returncode == 0, a.stderr[-3000:]
    assert "runtime error" not in a.stderr and "AddressSanitizer" not in a.stderr, a.stderr[-3000:]
    b = subprocess.run([plain], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=env, timeout=300)
    assert b.returncode == 0
    assert a.stdout == b.stdout and a.stdout.count("rc 0") == 21, a.stdout      # 7 cases x (fwd, block, reverse)


def test_pins_pass_under_ubsan():
    from oracle.build import build_sanitized
    build_sanitized()
    env = dict(os.environ, BIMAMBA_ORACLE_UBSAN="1", UBSAN_OPTIONS="halt_on_error=1")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env,
                       cwd=ROOT, timeout=600)
    assert r.returncode == 0, r.stdout[-3000:]
    assert "runtime error" not in r.stdout
