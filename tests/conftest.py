import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden(name):
    """Rows of a whitespace-separated golden file, comments stripped."""
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if line:
                rows.append(line.split())
    return rows


@pytest.fixture(scope="session")
def golden():
    return read_golden


# fp32-output tolerance of the two GEMV formulations (max_n |y - y*| / max_n |y*|): the lookup
# kernel accumulates exact table entries in fp32; the matrix core keeps 13 bits below the largest
# product of each 8-element run, so up to ~2^-13 of the products' magnitude can be lost.
GEMV_F32_TOL = {"lut": 2e-5, "mx": 2e-4}


@pytest.fixture(params=["lut", "mx"])
def gemv_path(request):
    """Forces one GEMV formulation for the test, yields its fp32-output tolerance."""
    from paper_2510_19482_amd import binding as B
    B.set_gemv_path(B.GEMV_LUT if request.param == "lut" else B.GEMV_MX)
    yield GEMV_F32_TOL[request.param]
    B.set_gemv_path(B.GEMV_AUTO)
