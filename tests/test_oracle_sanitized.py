"""The oracle's pins once more, against a build of the C oracle with gcc's
undefined-behaviour sanitizer (signed overflow, shifts, out-of-range
conversions, misaligned or null accesses trap on the first finding)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_pass_under_the_undefined_behaviour_sanitizer():
    env = dict(os.environ, ORACLE_SANITIZE="undefined")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                       text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-3000:]
    assert "runtime error" not in r.stdout
    assert os.path.exists(os.path.join(ROOT, "oracle", "liboracle_undefined.so"))
