"""Helpers shared by the GPU parity tests (no arithmetic of the method lives here)."""
import numpy as np

import oracle
from paper_1908_05460_amd import binding as B

TOL = {"fp32": 1e-4, "bf16": 2e-2}      # max |gpu - oracle| / max |oracle| per dW tensor
S_TOL = 1e-5                            # |S_gpu - S_oracle| <= S_TOL * sum |dY[n,k,:,:]|


def to_gpu(a):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a))
    if a.dtype == np.uint16:
        t = t.view(torch.bfloat16)
    return t.cuda()


def oracle_shape(d):
    return oracle.shape(d.N, d.C, d.H, d.W, d.K, d.R, d.S, d.stride_h, d.pad_h, d.stride_w, d.pad_w)


def as_float32(a):
    from paper_1908_05460_amd import inputs
    return inputs.bf16_bits_to_float32(a) if a.dtype == np.uint16 else a


def rand_inputs(d, seed, dtype="fp32", dy_std=0.01):
    """Same recipe as the workloads: X = relu(z), dY = std * z."""
    from paper_1908_05460_amd import inputs
    rng = np.random.default_rng(seed)
    X = np.maximum(rng.standard_normal((d.N, d.C, d.H, d.W), np.float32), 0)
    dY = rng.standard_normal((d.N, d.K, d.Ho, d.Wo), np.float32) * np.float32(dy_std)
    if dtype == "bf16":
        return inputs.float32_to_bf16_bits(X), inputs.float32_to_bf16_bits(dY)
    return X, dY


def normwise_err(got, want):
    scale = np.abs(want).max()
    return float(np.abs(got.astype(np.float64) - want).max() / (scale if scale > 0 else 1.0))


def elementwise_pass_rate(got, want, tol):
    """Share of entries with |g - o| <= tol*|o| + tol*rms(o): information beside the normwise bound."""
    want = np.asarray(want, np.float64)
    diff = np.abs(np.asarray(got, np.float64).reshape(want.shape) - want)
    rms = float(np.sqrt(np.mean(want * want)))
    return float(np.mean(diff <= tol * np.abs(want) + tol * rms))


def check_select(d, dY, idx_gpu, S_gpu):
    want_idx, want_S = oracle.select(oracle_shape(d), dY)
    assert np.array_equal(idx_gpu, want_idx), "selected positions differ from the oracle"
    bound = S_TOL * np.abs(as_float32(dY).astype(np.float64)).reshape(d.N, d.K, -1).sum(axis=2)
    assert np.all(np.abs(S_gpu.astype(np.float64) - want_S) <= bound + 1e-30), "map sums out of tolerance"
