"""The C ABI driven by a plain C++ program (HIP runtime only, no torch, no Python binding):
paper_2104_08542_amd/examples/abi_client.cpp, built by paper_2104_08542_amd/build.py.  It trains a
small table through a cache that evicts and compares the flushed table with a dense table updated on
the host."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

BIN = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                   "paper_2104_08542_amd", "examples", "abi_client")


@pytest.mark.parametrize("lookahead", [0, 1, 2, 3])
def test_plain_cpp_client_trains_through_the_c_abi(lookahead):
    assert os.path.exists(BIN), "examples/abi_client is not built: run python paper_2104_08542_amd/build.py"
    r = subprocess.run([BIN, str(lookahead)], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    assert "OK: lookahead %d, 0 mismatches" % lookahead in r.stdout
