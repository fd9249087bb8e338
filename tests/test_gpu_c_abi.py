"""The C ABI used from a plain C99 program (tests/c_abi/parity_main.c, built by
__graft_entry__.build()): HIP runtime for memory, no Python in the loop, every step compared with
the oracle inside the program."""
import os
import subprocess

import pytest

from tests.parity import log

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "tests", "c_abi", "parity_main")


@pytest.mark.gpu
@pytest.mark.parametrize("args", [
    ("1000003", "1024", "8", "0.005", "8"),
    ("300000", "96", "5", "0.01", "6"),          # a block size that is not a multiple of 256
])
def test_c_program_matches_the_oracle(args):
    if not os.path.exists(EXE):                 # a one-second gcc compile of one C file
        try:
            import __graft_entry__
            __graft_entry__.build_c_harness()
        except Exception as e:                  # no compiler on this machine
            pytest.skip(f"tests/c_abi/parity_main is not built and cannot be built here: {e}")
    r = subprocess.run([EXE, *args], capture_output=True, text=True, timeout=120)
    log(r.stdout[-600:])
    assert r.returncode == 0, r.stderr[-2000:]
    assert "c-abi parity ok" in r.stdout
    assert r.stdout.count(" ok\n") == int(args[4]) + 1


def test_c_program_usage_message():
    if not os.path.exists(EXE):
        pytest.skip("tests/c_abi/parity_main has not been built")
    r = subprocess.run([EXE], capture_output=True, text=True, timeout=30)
    assert r.returncode == 2 and "usage" in r.stderr
