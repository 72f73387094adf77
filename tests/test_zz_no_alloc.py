"""conv_wgrad_approx_static (the approximation on the library's own static scratch buffer, for callers that cannot
allocate) against conv_wgrad_approx and against the oracle: two calls in a row on the shared buffer, the second
on a smaller layer; then layers that take the other forms of the approximation; then the size limit."""
import ctypes

import numpy as np
import pytest

import oracle
from paper_1908_05460_amd import binding as B
from tests.gpu_util import TOL, check_select, normwise_err, oracle_shape, rand_inputs, to_gpu

pytestmark = pytest.mark.gpu


def run_both(d, seed, dtype="fp32", scale=1 / 128):
    """The new entry point through the C ABI, then the existing one on a caller workspace; returns both results."""
    import torch
    X, dY = rand_inputs(d, seed, dtype)
    Xg, dYg = to_gpu(X), to_gpu(dY)
    lib = B.load()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    dW = torch.full((d.K, d.C, d.R, d.S), float("nan"), device="cuda")
    idx = torch.full((d.N, d.K), -1, dtype=torch.int32, device="cuda")
    S = torch.full((d.N, d.K), float("nan"), device="cuda")
    rc = lib.conv_wgrad_approx_static(ctypes.byref(d), ctypes.c_void_p(Xg.data_ptr()), ctypes.c_void_p(dYg.data_ptr()),
                                      ctypes.c_void_p(dW.data_ptr()), ctypes.c_float(scale),
                                      ctypes.c_void_p(idx.data_ptr()), ctypes.c_void_p(S.data_ptr()), stream)
    assert rc == B.OK, B.load().conv_wgrad_status_string(rc)
    torch.cuda.synchronize()
    idx2 = torch.empty_like(idx); S2 = torch.empty_like(S)
    ref = B.conv_wgrad_approx(d, Xg, dYg, scale=scale, idx_out=idx2, sum_out=S2)
    torch.cuda.synchronize()
    got, ref = dW.cpu().numpy(), ref.cpu().numpy()
    # same kernels, same plan: positions bit-exact, dW identical (and inside the oracle's tolerance)
    assert np.array_equal(idx.cpu().numpy(), idx2.cpu().numpy())
    assert np.array_equal(S.cpu().numpy(), S2.cpu().numpy())
    assert np.isfinite(got).all()
    assert normwise_err(got, ref.astype(np.float64)) <= TOL[dtype]
    assert np.array_equal(got, ref)
    want, _, _ = oracle.wgrad_approx(oracle_shape(d), X, dY, scale=scale)
    check_select(d, dY, idx.cpu().numpy(), S.cpu().numpy())
    assert normwise_err(got, want) <= TOL[dtype]
    return got


def test_two_calls_in_a_row_the_second_smaller():
    big = B.desc(128, 256, 8, 8, 256)                  # LDS form: select + gather + reduction of 18 MiB of partials
    assert 16 << 20 < B.workspace_bytes(big, B.APPROX) <= B.STATIC_SCRATCH_BYTES
    run_both(big, 1)
    small = B.desc(16, 16, 32, 32, 16)                 # fused form, a few hundred KiB of the same buffer
    run_both(small, 2)
    run_both(big, 3)                                   # and the large one again over the small one's leftovers


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("shape", [(32, 3, 32, 32, 16), (64, 32, 16, 16, 64, 2), (32, 512, 2, 2, 512),
                                   (64, 128, 16, 16, 128), (7, 5, 9, 7, 6)])
def test_every_form_of_the_approximation(shape, dtype):
    N, C, H, W, K = shape[:5]
    stride = shape[5] if len(shape) > 5 else 1
    d = B.desc(N, C, H, W, K, stride=stride, dtype=B.BF16 if dtype == "bf16" else B.F32)
    run_both(d, N + C + K, dtype)


def test_a_layer_beyond_the_limit_is_refused_and_nothing_is_written():
    import torch
    d = B.desc(2048, 512, 4, 4, 512)
    assert B.workspace_bytes(d, B.APPROX) > B.STATIC_SCRATCH_BYTES
    dW = torch.full((512, 512, 3, 3), 7.0, device="cuda")
    x = torch.zeros(16, device="cuda")
    rc = B.load().conv_wgrad_approx_static(ctypes.byref(d), ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(x.data_ptr()),
                                           ctypes.c_void_p(dW.data_ptr()), ctypes.c_float(1.0), None, None, None)
    torch.cuda.synchronize()
    assert rc == B.SCRATCH_LIMIT
    assert bool((dW == 7.0).all())
