"""The oracle's pins once more, against builds of the C oracle with gcc's
sanitizers: undefined behaviour (signed overflow, shifts, out-of-range
conversions, misaligned or null accesses) and addresses (reads and writes
outside an array, on the heap, the stack or in globals).  Either stops at the
first finding.  Host code only."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run_pins(env):
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                           "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                          text=True, timeout=900)


def test_oracle_pins_pass_under_the_undefined_behaviour_sanitizer():
    r = _run_pins(dict(os.environ, ORACLE_SANITIZE="undefined"))
    assert r.returncode == 0, r.stdout[-3000:]
    assert "runtime error" not in r.stdout
    assert os.path.exists(os.path.join(ROOT, "oracle", "liboracle_undefined.so"))


def test_oracle_pins_pass_under_the_address_sanitizer():
    # the interpreter itself is not instrumented, so the sanitizer's runtime is loaded ahead of it (kept in front of
    # whatever is preloaded already); leak reports are off (the interpreter's own allocations are not the subject)
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    assert os.path.isabs(runtime) and os.path.exists(runtime), "gcc's address-sanitizer runtime not found"
    before = os.environ.get("LD_PRELOAD", "")
    env = dict(os.environ, ORACLE_SANITIZE="address,undefined",
               LD_PRELOAD=runtime + (":" + before if before else ""),
               ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:halt_on_error=1")
    r = _run_pins(env)
    assert r.returncode == 0, r.stdout[-3000:]
    assert "AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout
    assert os.path.exists(os.path.join(ROOT, "oracle", "liboracle_address_undefined.so"))
