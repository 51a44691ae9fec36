"""GPU test of the entry point that allocates nothing (ap_gemm_static) against ap_gemm.

Collected last (file name): a run with -x stops at the first failure, and a failure here must not hide other tests.
"""
import ctypes

import numpy as np
import pytest

import oracle
from paper_2402_10517_amd import inputs

pytestmark = pytest.mark.gpu
from gpu_util import tolerance


@pytest.fixture(scope="module")
def B():
    from paper_2402_10517_amd import binding
    return binding


def _both(B, torch, pm, b, x):
    """(ap_gemm_static output, ap_gemm output) through the raw C-ABI, with canaries around the first."""
    batch, M = x.shape[0], pm.M
    xd = torch.from_numpy(x).cuda()
    guard = 64
    ybuf = torch.full((guard + batch * M + guard,), -7.0, dtype=torch.float16, device="cuda")
    sp = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    st = B.lib.ap_gemm_static(pm.handle, b, xd.data_ptr(), ybuf.data_ptr() + 2 * guard, batch, sp)
    assert st == 0, B.strerror(st)
    y_ref = B.ap_gemm(pm, b, xd)
    torch.cuda.synchronize()
    out = ybuf.cpu().numpy()
    assert np.all(out[:guard] == -7.0) and np.all(out[-guard:] == -7.0)
    return out[guard:-guard].reshape(batch, M), y_ref.cpu().numpy()


def test_static_gemm_matches_gemm_on_two_calls_in_a_row(B):
    import torch
    # first call: larger matrix, ragged in every dimension (rows not a multiple of 16, batch not a
    # multiple of 16, a ragged last span); second call: a smaller matrix, which leaves the first
    # call's weights in the rest of the shared array
    cases = [((200, 2048 + 96, 37), (3, 8)), ((52, 160, 5), (4, 7))]
    for (M, K, batch), bits in cases:
        idx, luts, x = inputs.make_case(41, M, K, batch=batch)
        pm = B.ap_pack(idx, luts)
        for b in bits:
            got, ref = _both(B, torch, pm, b, x)
            _, mag = oracle.gemv(idx, luts[b], b, x)
            tol = tolerance(mag)
            err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
            assert np.all(np.isfinite(got))
            assert np.all(err <= 2 * tol), float(np.max(err / tol))   # each side is within tol of the exact value
            y_exact, _ = oracle.gemv(idx, luts[b], b, x)
            assert np.all(np.abs(got.astype(np.float64) - y_exact) <= tol)
        pm.close()


def test_static_gemm_rejects_what_does_not_fit(B):
    import torch
    sp = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    M, K = 4100, 4096                       # M*K*2 just above the 32 MiB array
    idx = np.zeros((M, K), dtype=np.uint8)
    lut = {3: np.zeros((M, 8), dtype=np.float16)}
    pm = B.ap_pack(idx, lut)
    x = torch.zeros((1, K), dtype=torch.float16, device="cuda")
    y = torch.zeros((1, M), dtype=torch.float16, device="cuda")
    assert B.lib.ap_gemm_static(pm.handle, 3, x.data_ptr(), y.data_ptr(), 1, sp) == 5
    assert B.lib.ap_gemm_static(pm.handle, 4, x.data_ptr(), y.data_ptr(), 1, sp) == 3
    assert B.lib.ap_gemm_static(pm.handle, 3, x.data_ptr(), y.data_ptr(), 0, sp) == 6
    assert B.lib.ap_gemm_static(pm.handle, 3, x.data_ptr() + 2, y.data_ptr(), 1, sp) == 1
    assert B.lib.ap_gemm_static(None, 3, x.data_ptr(), y.data_ptr(), 1, sp) == 1
    pm.close()
