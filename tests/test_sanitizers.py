"""Host-side sanitizer runs (no GPU, no device code instrumented):
  - the CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer on small shapes (oracle/sanitize_check.c);
  - the oracle pins against the oracle built with UndefinedBehaviorSanitizer;
  - the argument-validation tests of the C ABI against libxnor with UndefinedBehaviorSanitizer in csrc/api.hip.
Each instrumented build aborts (the host code of libxnor: traps) on its first finding, so a clean exit is the
assertion."""
import os
import subprocess
import sys

from oracle import build_oracle
from paper_1603_05279_amd import build as hip_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = build_oracle.build_sanitize_check(str(tmp_path / "sanitize_check"))
    r = subprocess.run([exe], capture_output=True, text=True, env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1"))
    assert r.returncode == 0, r.stderr[-4000:]
    assert "sanitize_check ok" in r.stdout


def test_oracle_pins_pass_against_the_ubsan_build_of_the_oracle():
    build_oracle.build(force=True, sanitize=True)
    env = dict(os.environ, XNOR_ORACLE_SANITIZE="1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")], capture_output=True, text=True, env=env,
                       cwd=ROOT)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert "runtime error" not in r.stdout + r.stderr


def test_abi_argument_checks_pass_against_the_ubsan_build_of_the_host_code(tmp_path):
    lib = hip_build.build_host_ubsan(str(tmp_path / "libxnor_ubsan.so"))
    env = dict(os.environ, XNOR_LIBRARY=lib, UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_abi.py")], capture_output=True, text=True, env=env, cwd=ROOT)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert "runtime error" not in r.stdout + r.stderr
