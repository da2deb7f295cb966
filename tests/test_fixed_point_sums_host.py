"""The fixed-point gradient sums of the matrix-core kernel (Eq. 9), checked on the host.

tests/host/check_fixed_point_sums.cpp is built with the plain C++ compiler against the header whose functions the kernel
calls (csrc/fixed_point_sums.h): the scale of a column, the bit pattern added for a term, the integer sum recovered
from a cell.  It checks the bounds of the scale, the rounding of single terms (ties, negative values), that cells which
wrap around give back the exact integer sum in any order of the additions, and the distance to the fp64 sum."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "tests", "host", "check_fixed_point_sums")


@pytest.fixture(scope="module")
def checker():
    src = os.path.join(ROOT, "tests", "host", "check_fixed_point_sums.cpp")
    inc = os.path.join(ROOT, "paper_1505_04956_amd", "csrc")
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-Wall", "-I", inc, "-o", EXE, src])
    yield EXE
    os.remove(EXE)


# mini-batch sizes of the workloads and the extremes the kernel admits, column maxima over many orders of magnitude
@pytest.mark.parametrize("b", [1, 2, 100, 255, 256, 1000, 2000, 4096, 65535])
@pytest.mark.parametrize("xmax", [1e-37, 1e-20, 0.001, 1.0, 13.7, 1000.5, 3e10])
def test_fixed_point_sums_are_exact_and_order_free(checker, b, xmax):
    out = subprocess.run([checker, str(b), repr(xmax), str(b % 97 + 1)], stdout=subprocess.PIPE, text=True)
    assert out.returncode == 0 and out.stdout.startswith("ok "), out.stdout
