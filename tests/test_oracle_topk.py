"""Pins for the oracle's top-k generalisation of the Max Gradient Approximation (CPU only).

Section 2.3 names the generalisation in one sentence and leaves its scaling open; the reading
of this build (every one of the k retained positions carries sum/k) is pinned by what must hold
under it: k = 1 is Algorithm 1; the result is the exact gradient of the k-sparse dY; with a
constant input and no padding it is x0 * sum for any k; k = map length is the exact gradient of
a map flattened to its mean.  The selection is pinned against a stable library sort.
"""
import numpy as np
import pytest

import oracle
from tests.test_oracle_exact import SHAPES, mk, rand_inputs


def sparsify_k(dY, idx, S):
    N, K, Ho, Wo = dY.shape
    k = idx.shape[2]
    out = np.zeros((N, K, Ho * Wo))
    nn, kk = np.meshgrid(np.arange(N), np.arange(K), indexing="ij")
    for j in range(k):
        out[nn, kk, idx[:, :, j]] += S / k
    return out.reshape(N, K, Ho, Wo)


@pytest.mark.parametrize("k", [1, 2, 3, 5])
def test_selection_is_a_stable_sort_by_decreasing_magnitude(k):
    g = oracle.shape(4, 2, 7, 6, 5, stride=1, pad=1)
    rng = np.random.default_rng(31 + k)
    dY = (rng.integers(-4, 5, size=(4, 5, 7, 6)) * 0.5).astype(np.float32)     # many equal magnitudes
    idx, S = oracle.select_topk(g, dY, k)
    flat = np.abs(dY.astype(np.float64)).reshape(4, 5, -1)
    want = np.argsort(-flat, axis=2, kind="stable")[:, :, :k]                   # ties: lower index first
    assert np.array_equal(idx, want)
    np.testing.assert_allclose(S, dY.astype(np.float64).reshape(4, 5, -1).sum(axis=2), atol=1e-12)


def test_k_equal_one_is_algorithm_1():
    for t in SHAPES[:4]:
        g = mk(t)
        X, dY = rand_inputs(g, 77, np.float32)
        a, ia, Sa = oracle.wgrad_approx(g, X, dY, scale=0.5)
        b, ib, Sb = oracle.wgrad_approx_topk(g, X, dY, 1, scale=0.5)
        assert np.array_equal(a, b) and np.array_equal(ia, ib[:, :, 0]) and np.array_equal(Sa, Sb)


@pytest.mark.parametrize("k", [2, 4])
@pytest.mark.parametrize("t", SHAPES[:5])
def test_topk_is_the_exact_gradient_of_the_k_sparse_dY(t, k):
    g = mk(t)
    Ho, Wo = oracle.out_hw(g)
    if Ho * Wo < k:
        pytest.skip("map shorter than k")
    X, dY = rand_inputs(g, 5, np.float32)
    dW, idx, S = oracle.wgrad_approx_topk(g, X, dY, k)
    want = oracle.wgrad_exact(g, X.astype(np.float64), sparsify_k(dY, idx, S))
    np.testing.assert_allclose(dW, want, rtol=1e-12, atol=1e-14 * np.abs(want).max())
    # k retained entries per map: sparsity 1 - k/(Ho*Wo) (Section 2.3 states 1 - 1/(HW) for k = 1)
    assert (sparsify_k(dY, idx, S) != 0).sum() <= g.N * g.K * k


@pytest.mark.parametrize("k", [1, 3, 6])
def test_constant_input_without_padding_gives_x0_times_the_sums(k):
    g = oracle.shape(3, 2, 6, 5, 4, R=3, S=2, stride=1, pad=0)
    _, dY = rand_inputs(g, 9, np.float32)
    X = np.full((3, 2, 6, 5), 1.25, np.float32)
    dW, _, S = oracle.wgrad_approx_topk(g, X, dY, k, scale=2.0)
    want = 2.0 * 1.25 * S.sum(axis=0)                        # per output channel, every (c, r, s) alike
    np.testing.assert_allclose(dW, np.broadcast_to(want[:, None, None, None], dW.shape), rtol=1e-12)


def test_k_equal_map_length_is_the_exact_gradient_of_the_mean_map():
    g = oracle.shape(2, 3, 4, 4, 2, stride=1, pad=1)
    X, dY = rand_inputs(g, 13, np.float32)
    L = 16
    dW, idx, S = oracle.wgrad_approx_topk(g, X, dY, L)
    assert np.array_equal(np.sort(idx, axis=2), np.broadcast_to(np.arange(L), idx.shape))   # every position once
    mean_map = np.broadcast_to((S / L)[:, :, None, None], dY.shape)
    want = oracle.wgrad_exact(g, X.astype(np.float64), np.ascontiguousarray(mean_map))
    np.testing.assert_allclose(dW, want, rtol=1e-12, atol=1e-14 * np.abs(want).max())


def test_k_out_of_range_is_refused():
    g = oracle.shape(1, 1, 2, 2, 1, stride=1, pad=1)
    dY = np.zeros((1, 1, 2, 2), np.float32)
    for k in (0, 5):
        with pytest.raises(AssertionError):
            oracle.select_topk(g, dY, k)
