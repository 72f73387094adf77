"""Pins for the oracle's exact filter gradient (CPU only).

Every check compares the oracle with something that is not the oracle: an
independently formulated forward convolution (pad + strided slices + einsum),
a library GEMM, a library autograd, or an algebraic property.
"""
import numpy as np
import pytest

import oracle

SHAPES = [
    # N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w
    (2, 3, 5, 5, 2, 3, 3, 1, 1, 1, 1),
    (2, 3, 5, 5, 2, 3, 3, 1, 1, 0, 0),
    (2, 3, 6, 5, 2, 3, 3, 2, 2, 1, 1),
    (2, 2, 7, 6, 3, 3, 2, 2, 1, 1, 0),   # non-square everything: catches swapped h/w, r/s
    (3, 2, 6, 7, 2, 2, 3, 1, 2, 0, 2),
    (1, 1, 4, 4, 1, 1, 1, 1, 1, 0, 0),
    (2, 2, 8, 8, 2, 5, 5, 1, 1, 2, 2),
]


def mk(shape_tuple):
    N, C, H, W, K, R, S, sh, sw, ph, pw = shape_tuple
    return oracle.shape(N, C, H, W, K, R, S, stride=sh, pad=ph, stride_w=sw, pad_w=pw)


def rand_inputs(g, seed, dtype=np.float64):
    rng = np.random.default_rng(seed)
    Ho, Wo = oracle.out_hw(g)
    X = rng.standard_normal((g.N, g.C, g.H, g.W)).astype(dtype)
    dY = rng.standard_normal((g.N, g.K, Ho, Wo)).astype(dtype)
    return X, dY


def forward_conv(g, X, Wt):
    """Y[n,k,h,w] = sum_{c,r,s} Wt[k,c,r,s] * Xpad[n,c,h*sh+r, w*sw+s]; formulated with
    explicit zero padding and strided slices, not with index arithmetic per element."""
    Ho, Wo = oracle.out_hw(g)
    Xp = np.pad(X.astype(np.float64), ((0, 0), (0, 0), (g.pad_h, g.pad_h), (g.pad_w, g.pad_w)))
    Y = np.zeros((g.N, g.K, Ho, Wo))
    for r in range(g.R):
        for s in range(g.S):
            win = Xp[:, :, r:r + g.stride_h * (Ho - 1) + 1:g.stride_h,
                     s:s + g.stride_w * (Wo - 1) + 1:g.stride_w]
            Y += np.einsum("kc,nchw->nkhw", Wt[:, :, r, s], win)
    return Y


@pytest.mark.parametrize("st", SHAPES)
def test_exact_equals_linear_functional_on_unit_filters(st):
    """L(W) = sum(dY * conv(X, W)) is linear in W, so dL/dW[k,c,r,s] = L(e_kcrs) exactly;
    brute force over every filter entry."""
    g = mk(st)
    X, dY = rand_inputs(g, 11)
    dW = oracle.wgrad_exact(g, X, dY)
    for k in range(g.K):
        for c in range(g.C):
            for r in range(g.R):
                for s in range(g.S):
                    E = np.zeros((g.K, g.C, g.R, g.S))
                    E[k, c, r, s] = 1.0
                    want = float(np.sum(dY * forward_conv(g, X, E)))
                    assert dW[k, c, r, s] == pytest.approx(want, rel=1e-12, abs=1e-12)


@pytest.mark.parametrize("st", SHAPES)
def test_exact_matches_library_autograd(st):
    import torch
    g = mk(st)
    X, dY = rand_inputs(g, 5)
    Wt = torch.zeros(g.K, g.C, g.R, g.S, dtype=torch.float64, requires_grad=True)
    Y = torch.nn.functional.conv2d(torch.from_numpy(X), Wt, stride=(g.stride_h, g.stride_w),
                                   padding=(g.pad_h, g.pad_w))
    (Y * torch.from_numpy(dY)).sum().backward()
    np.testing.assert_allclose(oracle.wgrad_exact(g, X, dY), Wt.grad.numpy(), rtol=1e-11, atol=1e-11)


def test_zero_dY_gives_exact_zero():
    g = mk(SHAPES[0])
    X, dY = rand_inputs(g, 1)
    assert np.all(oracle.wgrad_exact(g, X, np.zeros_like(dY)) == 0.0)


def test_one_by_one_filter_is_a_plain_gemm():
    g = oracle.shape(4, 5, 6, 7, 3, R=1, S=1, stride=1, pad=0)
    X, dY = rand_inputs(g, 2)
    want = dY.transpose(1, 0, 2, 3).reshape(g.K, -1) @ X.transpose(1, 0, 2, 3).reshape(g.C, -1).T
    np.testing.assert_allclose(oracle.wgrad_exact(g, X, dY)[:, :, 0, 0], want, rtol=1e-12, atol=1e-12)


def test_bilinear_and_batch_permutation_invariant():
    g = mk(SHAPES[3])
    X1, dY1 = rand_inputs(g, 3)
    X2, dY2 = rand_inputs(g, 4)
    f = oracle.wgrad_exact
    np.testing.assert_allclose(f(g, 2 * X1 - 3 * X2, dY1), 2 * f(g, X1, dY1) - 3 * f(g, X2, dY1), atol=1e-11)
    np.testing.assert_allclose(f(g, X1, dY1 + 0.5 * dY2), f(g, X1, dY1) + 0.5 * f(g, X1, dY2), atol=1e-11)
    perm = np.array([1, 0])
    np.testing.assert_allclose(f(g, X1[perm], dY1[perm]), f(g, X1, dY1), atol=1e-12)


def test_stride_two_equals_stride_one_with_zero_upsampled_dY():
    g2 = oracle.shape(2, 2, 8, 8, 3, stride=2, pad=1)
    X, dY = rand_inputs(g2, 6)
    g1 = oracle.shape(2, 2, 8, 8, 3, stride=1, pad=1)
    Ho1, Wo1 = oracle.out_hw(g1)
    up = np.zeros((2, 3, Ho1, Wo1))
    up[:, :, ::2, ::2] = dY
    np.testing.assert_allclose(oracle.wgrad_exact(g2, X, dY), oracle.wgrad_exact(g1, X, up), atol=1e-12)


def test_single_impulse_reads_the_right_input_element():
    """dY one-hot at (n,k,h,w) and X one-hot at (n,c,ih,iw): dW is 1 exactly at the tap
    with ih = h*sh + r - ph and iw = w*sw + s - pw, and 0 elsewhere."""
    g = mk(SHAPES[3])
    Ho, Wo = oracle.out_hw(g)
    n, k, h, w, c, r, s = 1, 2, 2, 3, 1, 2, 1
    ih, iw = h * g.stride_h + r - g.pad_h, w * g.stride_w + s - g.pad_w
    assert 0 <= ih < g.H and 0 <= iw < g.W
    X = np.zeros((g.N, g.C, g.H, g.W)); X[n, c, ih, iw] = 1.0
    dY = np.zeros((g.N, g.K, Ho, Wo)); dY[n, k, h, w] = 1.0
    want = np.zeros((g.K, g.C, g.R, g.S)); want[k, c, r, s] = 1.0
    assert np.array_equal(oracle.wgrad_exact(g, X, dY), want)


def test_sampled_entries_agree_with_full_tensor():
    g = mk(SHAPES[2])
    X, dY = rand_inputs(g, 8, np.float32)
    full = oracle.wgrad_exact(g, X, dY).ravel()
    pick = np.array([0, 5, 17, full.size - 1])
    assert np.array_equal(oracle.wgrad_exact_at(g, X, dY, pick), full[pick])


def test_float32_and_bf16_inputs_are_upcast_exactly():
    from paper_1908_05460_amd import inputs
    g = mk(SHAPES[0])
    X, dY = rand_inputs(g, 9, np.float32)
    assert np.array_equal(oracle.wgrad_exact(g, X, dY),
                          oracle.wgrad_exact(g, X.astype(np.float64), dY.astype(np.float64)))
    Xb, dYb = inputs.float32_to_bf16_bits(X), inputs.float32_to_bf16_bits(dY)
    Xf, dYf = inputs.bf16_bits_to_float32(Xb), inputs.bf16_bits_to_float32(dYb)
    assert np.array_equal(oracle.wgrad_exact(g, Xb, dYb), oracle.wgrad_exact(g, Xf, dYf))
    # the bit trick used above is the rounding torch performs
    import torch
    assert np.array_equal(Xf, torch.from_numpy(X).to(torch.bfloat16).float().numpy())
