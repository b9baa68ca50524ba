"""The oracle's C source under the undefined-behaviour sanitizer: built with
-fsanitize=undefined,bounds-strict,float-cast-overflow (no recovery) and run through the oracle's own
CPU pins in a child process.  An out-of-bounds index, a signed overflow in an index product, a
misaligned or null access or a float-to-int conversion out of range aborts the child."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "easyspec_oracle.c")
PINS = ["tests/test_oracle_pins.py", "tests/test_oracle_tree.py", "tests/test_oracle_accept.py",
        "tests/test_oracle_full_layer.py", "tests/test_oracle_rounding.py"]


def test_oracle_pins_pass_under_the_undefined_behaviour_sanitizer(tmp_path):
    so = str(tmp_path / "libeasyspec_oracle_ubsan.so")
    cc = subprocess.run(["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall",
                         "-fsanitize=undefined,bounds-strict,float-cast-overflow", "-fno-sanitize-recover=all",
                         "-o", so, SRC, "-lm"], capture_output=True, text=True)
    if cc.returncode != 0 and "ubsan" in (cc.stderr + cc.stdout).lower():
        pytest.skip("no sanitizer runtime for gcc on this machine")
    assert cc.returncode == 0, cc.stderr[-2000:]
    env = dict(os.environ, EASYSPEC_ORACLE_LIB=so, UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    p = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-k", "not sanitizer", *PINS],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (p.stdout + p.stderr)[-3000:]
    assert p.returncode == 0, tail
    assert "runtime error" not in p.stdout + p.stderr, tail
    assert " passed" in p.stdout
