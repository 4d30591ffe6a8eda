"""The entry point that allocates nothing (qg_gemv_noalloc: the library's own scratch array in
place of a caller's workspace), called through the C-ABI and compared bit for bit with qg_gemv on
the same inputs -- same kernels, same split of K, so the same bits."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2307_03738_amd import synth
from tests.util import dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qg():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2307_03738_amd import binding
    binding.lib()
    return binding


def _problem(qg, seed, N, K, bits, group):
    W, x = synth.small_case(seed, N, K, 0.02, True)
    q, s, z = qg.qg_quantize(dev(W), bits, group)
    return qg.qg_pack(q, s, z, bits, group), dev(x)


def _both(qg, blob, x, N, K, bits, group):
    """(y of qg_gemv with a caller's workspace, y of qg_gemv_noalloc), raw C calls."""
    L = qg.lib()
    stream = torch.cuda.current_stream().cuda_stream
    ws = qg.new_workspace(qg.qg_workspace_bytes(N, K, bits, group, 1))
    y_ref = torch.full((N,), 3.0, dtype=torch.float32, device="cuda")
    y = torch.full((N + 64,), 7.0, dtype=torch.float32, device="cuda")          # canary behind y
    rc = L.qg_gemv(blob.data_ptr(), N, K, bits, group, x.data_ptr(), y_ref.data_ptr(), ws.data_ptr(),
                   ws.numel(), stream)
    assert rc == 0, rc
    rc = L.qg_gemv_noalloc(blob.data_ptr(), N, K, bits, group, x.data_ptr(), y.data_ptr(), stream)
    assert rc == 0, rc
    torch.cuda.synchronize()
    yh = host(y)
    assert np.all(yh[N:] == 7.0), "write past the end of y"
    return host(y_ref), yh[:N]


# K cut over workgroups (the scratch is what the partial sums meet in), then a smaller problem
# whose slots are a subset of the ones the first call used
@pytest.mark.parametrize("first,second", [
    ((200, 11008, 4, 128), (70, 4096, 4, 128)),
    ((130, 11008, 3, 11008), (64, 512, 3, 64)),
    ((300, 8192, 2, 32), (130, 8192, 2, 32)),
])
def test_noalloc_matches_gemv_on_two_calls_in_a_row(qg, first, second):
    qg.qg_set_gemv_tuning(2, 4096, 0)          # short wavefronts: every tile's K is cut over several workgroups
    try:
        for i, (N, K, bits, group) in enumerate((first, second)):
            print("[case] noalloc", N, K, bits, group, flush=True)
            blob, x = _problem(qg, 5000 + i + N, N, K, bits, group)
            y_ref, y = _both(qg, blob, x, N, K, bits, group)
            assert np.array_equal(y_ref.view(np.uint32), y.view(np.uint32))
            assert np.isfinite(y).all()
    finally:
        qg.qg_set_gemv_tuning(0, 0, 0)


def test_noalloc_built_in_launch_shape(qg):
    for N, K, bits, group in ((4096, 11008, 4, 128), (512, 512, 4, 64)):
        print("[case] noalloc default shape", N, K, bits, group, flush=True)
        blob, x = _problem(qg, 5100 + N, N, K, bits, group)
        y_ref, y = _both(qg, blob, x, N, K, bits, group)
        assert np.array_equal(y_ref.view(np.uint32), y.view(np.uint32))


def test_noalloc_refuses_what_does_not_fit_and_bad_arguments(qg):
    L = qg.lib()
    stream = torch.cuda.current_stream().cuda_stream
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    too_many = 63488 + 1                       # QG_NOALLOC_MAX_N + 1
    assert L.qg_gemv_noalloc(buf.data_ptr(), too_many, 128, 4, 128, buf.data_ptr(), buf.data_ptr(), stream) == 5
    assert L.qg_gemv_noalloc(None, 64, 128, 4, 128, buf.data_ptr(), buf.data_ptr(), stream) == 1
    assert L.qg_gemv_noalloc(buf.data_ptr(), 64, 100, 4, 128, buf.data_ptr(), buf.data_ptr(), stream) == 2
    assert L.qg_gemv_noalloc(buf.data_ptr(), 64, 128, 4, 128, buf.data_ptr() + 4, buf.data_ptr(), stream) == 4
    torch.cuda.synchronize()
    assert not host(buf).any()                 # nothing was enqueued
