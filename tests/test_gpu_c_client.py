"""The library called from a plain C program (tests/c_client/zeco_c_client.c): three calls and the fused
forward on a segment length that is no multiple of 64, checked inside the program against the C oracle."""
import os
import subprocess
import sys

import pytest

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_client"))
import build_c_client as c_client_build   # noqa: E402


def test_c_client_builds_against_the_header():
    """gcc -std=c11 -pedantic accepts include/zeco.h and the program links against libzeco.so (no GPU needed)."""
    from paper_2507_01004_amd import zeco
    zeco.lib()                                   # the library the client links is there
    exe = c_client_build.build(force=True)
    assert os.access(exe, os.X_OK)


@pytest.mark.gpu
def test_c_client_matches_the_oracle():
    exe = c_client_build.build(force=False)
    print("running", exe, flush=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=100)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0 and r.stdout.strip().endswith("OK")
