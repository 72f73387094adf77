"""Pins of the oracle's channel-last functions (the layouts of the paper's own kernel, Section 2.4:
X[n,h,w,c], dY[n,k,h,w], dW as [k,r,s,c] or [r,s,c,k]).  They index the channel-last tensors with
loops of their own, so each pin below would catch a swapped axis or a wrong stride in them."""
import numpy as np
import pytest

import oracle

SHAPES = [
    # N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w
    (2, 3, 5, 4, 2, 3, 3, 1, 1, 1, 1),
    (3, 4, 6, 7, 5, 3, 2, 2, 1, 1, 0),       # every extent different, mixed stride and padding
    (2, 5, 4, 4, 3, 1, 1, 1, 1, 0, 0),
    (1, 2, 7, 5, 3, 5, 3, 1, 2, 2, 1),
]


def shape_of(t):
    N, C, H, W, K, R, S, sh, sw, ph, pw = t
    return oracle.shape(N, C, H, W, K, R, S, stride=sh, pad=ph, stride_w=sw, pad_w=pw)


def rand(t, seed):
    g = shape_of(t)
    Ho, Wo = oracle.out_hw(g)
    rng = np.random.default_rng(seed)
    return g, rng.standard_normal((g.N, g.C, g.H, g.W)), rng.standard_normal((g.N, g.K, Ho, Wo))


def brute_force_exact_nhwc(g, Xl, dY):
    """dW[k,r,s,c] straight from the definition, python loops over the output, on X[n,h,w,c]."""
    Ho, Wo = oracle.out_hw(g)
    Xp = np.zeros((g.N, g.H + 2 * g.pad_h, g.W + 2 * g.pad_w, g.C))
    Xp[:, g.pad_h:g.pad_h + g.H, g.pad_w:g.pad_w + g.W, :] = Xl
    dW = np.zeros((g.K, g.R, g.S, g.C))
    for n in range(g.N):
        for h in range(Ho):
            for w in range(Wo):
                window = Xp[n, h * g.stride_h:h * g.stride_h + g.R, w * g.stride_w:w * g.stride_w + g.S, :]   # [R,S,C]
                dW += dY[n, :, h, w][:, None, None, None] * window[None]
    return dW


@pytest.mark.parametrize("t", SHAPES)
def test_exact_nhwc_equals_the_definition_by_brute_force(t):
    g, X, dY = rand(t, 1)
    Xl = oracle.x_to_nhwc(X)
    want = brute_force_exact_nhwc(g, Xl, dY)
    got = oracle.wgrad_exact_nhwc(g, Xl, dY, oracle.OHWI)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
    assert np.allclose(oracle.wgrad_exact_nhwc(g, Xl, dY, oracle.HWIO), want.transpose(1, 2, 3, 0), rtol=1e-12, atol=1e-12)
    assert np.allclose(oracle.wgrad_exact_nhwc(g, Xl, dY, oracle.OIHW), want.transpose(0, 3, 1, 2), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("t", SHAPES)
def test_channel_last_route_equals_the_nchw_route(t):
    # two independently indexed implementations of one definition, joined by a library transpose
    g, X, dY = rand(t, 2)
    Xl = oracle.x_to_nhwc(X)
    ex = oracle.wgrad_exact(g, X, dY)
    ap, idx, S = oracle.wgrad_approx(g, X, dY, scale=0.25)
    for layout, perm in ((oracle.OIHW, (0, 1, 2, 3)), (oracle.OHWI, (0, 2, 3, 1)), (oracle.HWIO, (2, 3, 1, 0))):
        assert np.allclose(oracle.wgrad_exact_nhwc(g, Xl, dY, layout), ex.transpose(perm), rtol=1e-12, atol=1e-12)
        ap2, idx2, S2 = oracle.wgrad_approx_nhwc(g, Xl, dY, scale=0.25, dw_layout=layout)
        assert np.allclose(ap2, ap.transpose(perm), rtol=1e-12, atol=1e-12)
        assert np.array_equal(idx2, idx) and np.array_equal(S2, S)


def test_an_input_that_encodes_its_own_coordinates_lands_where_the_layout_says():
    # X[n,h,w,c] = 1000 n + 100 h + 10 w + c and one-hot maps: every dW entry is one known element of X
    g = oracle.shape(2, 4, 6, 5, 3, 3, 3, stride=1, pad=1)
    Ho, Wo = oracle.out_hw(g)
    n_, h_, w_, c_ = np.meshgrid(np.arange(g.N), np.arange(g.H), np.arange(g.W), np.arange(g.C), indexing="ij")
    Xl = (1000 * n_ + 100 * h_ + 10 * w_ + c_).astype(np.float64)
    dY = np.zeros((g.N, g.K, Ho, Wo))
    spots = {0: (2, 3), 1: (0, 0), 2: (5, 4)}            # interior, top-left corner, bottom-right corner
    for k, (h, w) in spots.items():
        dY[1, k, h, w] = 2.0                             # image 1 only; image 0 stays zero
    for fn in (lambda L: oracle.wgrad_exact_nhwc(g, Xl, dY, L), lambda L: oracle.wgrad_approx_nhwc(g, Xl, dY, 1.0, L)[0]):
        ohwi, hwio = fn(oracle.OHWI), fn(oracle.HWIO)
        assert ohwi.shape == (3, 3, 3, 4) and hwio.shape == (3, 3, 4, 3)
        for k, (h, w) in spots.items():
            for r in range(3):
                for s in range(3):
                    ih, iw = h + r - 1, w + s - 1
                    inside = 0 <= ih < g.H and 0 <= iw < g.W
                    for c in range(g.C):
                        want = 2.0 * (1000 + 100 * ih + 10 * iw + c) if inside else 0.0
                        assert ohwi[k, r, s, c] == want and hwio[r, s, c, k] == want


def test_layout_helpers_against_explicit_loops():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((2, 3, 4, 5))
    Xl = oracle.x_to_nhwc(X)
    assert Xl.shape == (2, 4, 5, 3) and Xl.flags["C_CONTIGUOUS"]
    for n in range(2):
        for c in range(3):
            for h in range(4):
                for w in range(5):
                    assert Xl[n, h, w, c] == X[n, c, h, w]
    assert np.array_equal(oracle.x_to_nchw(Xl), X)
    dW = rng.standard_normal((6, 3, 2, 4))               # K, C, R, S
    ohwi = oracle.dw_permute(dW, oracle.OIHW, oracle.OHWI)
    hwio = oracle.dw_permute(dW, oracle.OIHW, oracle.HWIO)
    assert ohwi.shape == (6, 2, 4, 3) and hwio.shape == (2, 4, 3, 6)
    for k in range(6):
        for c in range(3):
            for r in range(2):
                for s in range(4):
                    assert ohwi[k, r, s, c] == dW[k, c, r, s] and hwio[r, s, c, k] == dW[k, c, r, s]
    for a in (oracle.OIHW, oracle.OHWI, oracle.HWIO):
        for b in (oracle.OIHW, oracle.OHWI, oracle.HWIO):
            there = oracle.dw_permute(dW, oracle.OIHW, a)
            assert np.array_equal(oracle.dw_permute(oracle.dw_permute(there, a, b), b, oracle.OIHW), dW)
    assert np.array_equal(oracle.dw_permute(ohwi, oracle.OHWI, oracle.HWIO), hwio)     # the paper's second transpose


def test_bf16_and_fp32_inputs_are_widened_exactly():
    g, X, dY = rand(SHAPES[0], 4)
    from paper_1908_05460_amd import inputs
    Xb, dYb = inputs.float32_to_bf16_bits(X.astype(np.float32)), inputs.float32_to_bf16_bits(dY.astype(np.float32))
    Xw, dYw = inputs.bf16_bits_to_float32(Xb).astype(np.float64), inputs.bf16_bits_to_float32(dYb).astype(np.float64)
    a = oracle.wgrad_exact_nhwc(g, oracle.x_to_nhwc(Xb), dYb)
    b = oracle.wgrad_exact_nhwc(g, oracle.x_to_nhwc(Xw), dYw)
    assert np.array_equal(a, b)
