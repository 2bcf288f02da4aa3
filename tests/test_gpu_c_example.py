"""The C ABI called from plain C (no Python, no torch): paper_2412_01152_amd/csrc/example_outer_sync.c
runs one outer synchronisation and checks, on the host, what the definitions fix exactly.  The
executable is built next to the library by `python -m paper_2412_01152_amd.build`."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))
EXE = os.path.join(os.path.dirname(HERE), "paper_2412_01152_amd", "example_outer_sync")


def test_plain_c_caller_runs_an_outer_synchronisation():
    if not os.path.exists(EXE):                      # host compile of one C file against the built library
        from paper_2412_01152_amd import build
        build.build_example()
    r = subprocess.run([EXE], capture_output=True, text=True, timeout=110)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.strip().endswith("OK")
