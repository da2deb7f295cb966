"""The entry point that allocates nothing (Eq. 8 with its scratch in a static device array) against asgd_quant_error(),
through the C ABI: two calls in a row, the second with a smaller input, for the three Eq. 8 kernels."""
import numpy as np
import pytest

from paper_1505_04956_amd import workloads

pytestmark = pytest.mark.gpu


def make_data(N, d, k, seed):
    wl = workloads.Workload("t", N, d, k, 1, 1, 0.1, 0, 1, 1.0, "uniform10", "equal", data_seed=seed)
    return workloads.generate_host(wl)


@pytest.mark.parametrize("k,d,N1,N2", [
    (10, 10, 300_007, 4_001),       # streaming kernel
    (64, 32, 50_000, 777),          # matrix-core kernel
    (7, 5, 20_003, 64),             # generic kernel
])
def test_no_alloc_entry_point_matches_quant_error(k, d, N1, N2):
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device; there is no CPU fallback")
    from paper_1505_04956_amd import binding as B
    stream = torch.cuda.current_stream().cuda_stream
    out = torch.zeros(1, dtype=torch.float64, device="cuda:0")
    for N in (N1, N2):                                   # the second call is smaller: stale partial sums must not leak in
        X = torch.from_numpy(make_data(N, d, k, seed=N % 97)).to("cuda:0")
        g = B.ASGD(k, d, 1, min(N, 64), 0.05)
        g.load_shards(X)
        g.run_steps(3)                                   # some state other than the first k rows
        want = g.quant_error(0)
        w = torch.from_numpy(g.get_state(0)).to("cuda:0")
        out.fill_(-1.0)
        B.asgd_quant_error_noalloc(X.data_ptr(), N, k, d, w.data_ptr(), out.data_ptr(), stream)
        torch.cuda.synchronize()
        got = float(out.cpu()[0])
        assert got == want, (N, got, want)               # same kernels, same order of summation: bit for bit
        g.close()
    # arguments beyond the limits are refused, nothing is enqueued
    lib = B.lib()
    assert lib.asgd_quant_error_noalloc(X.data_ptr(), (1 << 40) + 1, k, d, w.data_ptr(), out.data_ptr(), stream) == B.EINVAL
    assert lib.asgd_quant_error_noalloc(X.data_ptr(), N, 1 << 13, 1 << 12, w.data_ptr(), out.data_ptr(), stream) == B.EINVAL
    assert lib.asgd_quant_error_noalloc(None, N, k, d, w.data_ptr(), out.data_ptr(), stream) == B.EINVAL
