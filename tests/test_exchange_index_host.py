"""Every offset the plain-row kernels form in the exchange buffers, and the LDS layout of the matrix-core kernel,
checked on the host for the full-size shapes.

tests/host/check_exchange_index.cpp is built with the plain C++ compiler against the header whose functions the
kernels call (csrc/exchange_index.h): schedule, buffer index, part of a partial message, rows of a part.  It walks all
rounds of a run of 80 epochs, all workers and copies, and checks every index against the sizes asgd_create allocates, that sender
and recipient agree on buffer and parity, that the recipient waits for the worker that actually sends, and that the
deterministic schedule fills every buffer exactly once per round."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "tests", "host", "check_exchange_index")


@pytest.fixture(scope="module")
def checker():
    src = os.path.join(ROOT, "tests", "host", "check_exchange_index.cpp")
    inc = os.path.join(ROOT, "paper_1505_04956_amd", "csrc")
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-Wall", "-I", inc, "-o", EXE, src])
    yield EXE
    os.remove(EXE)


# (k, d, W, E, steps per epoch, b) of the wider and the contraction workload, 80 epochs each
SHAPES = {"cfg2_wider": (100, 100, 512, 8, 19, 2000), "cfg4_contraction": (1024, 128, 256, 4, 4, 4096),
          "tiny": (7, 4, 5, 1, 50, 33)}


@pytest.mark.parametrize("shape", sorted(SHAPES))
@pytest.mark.parametrize("nb,parts", [(1, 1), (1, 4), (1, 16), (4, 4), (4, 1), (3, 7)])
def test_every_exchange_offset_is_inside_its_allocation(checker, shape, nb, parts):
    k, d, W, E, S, b = SHAPES[shape]
    if parts > k or nb > W - 1:
        pytest.skip("more parts than rows or more copies than other workers")
    rounds = 80 * S // E
    out = subprocess.run([checker, str(k), str(d), str(W), str(nb), str(parts), str(rounds), "1", str(b)],
                         stdout=subprocess.PIPE, text=True)
    assert out.returncode == 0 and out.stdout.startswith("ok "), out.stdout
    assert int(out.stdout.split()[1]) > rounds * W * nb
