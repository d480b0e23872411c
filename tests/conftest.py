import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    # the tests load the library that is built; only a tree with nothing built compiles it here
    # (hipcc cross-compiles for gfx950 without a GPU).  The build script is loaded by path:
    # importing the package needs the library.
    lib = os.path.join(ROOT, "paper_2104_08542_amd", "libsfc.so")
    client = os.path.join(ROOT, "paper_2104_08542_amd", "examples", "abi_client")
    if not os.path.exists(lib) or not os.path.exists(client):
        import importlib.util
        spec = importlib.util.spec_from_file_location(
            "sfc_hip_build", os.path.join(ROOT, "paper_2104_08542_amd", "build.py"))
        mod = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(mod)
        if not os.path.exists(lib):
            mod.build()
        mod.build_example()


def read_golden(name):
    """Parse 'key: v v v' lines of a golden text fixture into {key: [str, ...]}."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split(":", 1)
            out[k.strip()] = v.split()
    return out


def golden_ints(name):
    return {k: [int(x) for x in v] if all("," not in x for x in v) else v
            for k, v in read_golden(name).items()}


@pytest.fixture(scope="session")
def golden():
    return golden_ints
