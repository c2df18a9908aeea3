"""The oracle's pins once more, on its -fsanitize=address,undefined build: an out-of-bounds index, a read of
uninitialised stack, a signed overflow or a misaligned access in the plain C loops would otherwise pass
unnoticed as long as the numbers come out right.  Runs in a child interpreter that starts with the sanitizer
runtime preloaded (an instrumented shared object cannot be loaded into a process that started without it)."""
import os
import subprocess
import sys

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["tests/test_oracle_pins.py", "tests/test_lsh_oracle_pins.py", "tests/test_bea_oracle_pins.py",
             "tests/test_user_oracle_pins.py"]


def test_pins_pass_on_the_sanitized_oracle():
    oracle.build(sanitize=True)
    env = oracle.sanitizer_env()
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PIN_FILES],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert " passed" in r.stdout, tail
    # the child really ran the instrumented library
    probe = subprocess.run([sys.executable, "-c",
                            "import oracle, sys; oracle.lib(); "
                            "sys.exit(0 if any('libaif_oracle_san' in l for l in open('/proc/self/maps')) else 3)"],
                           cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert probe.returncode == 0, probe.stderr[-2000:]
