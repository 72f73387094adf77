"""GPU parity of the channel-last entry points (the layouts of the paper's own kernel, Section 2.4),
through the C ABI, against the oracle's channel-last functions; the two stand-alone transposes
are byte-exact against the oracle's definitions."""
import numpy as np
import pytest

import oracle
from paper_1908_05460_amd import binding as B, inputs
from tests.gpu_util import TOL, check_select, normwise_err, oracle_shape, rand_inputs, to_gpu
from tests.test_gpu_parity import SMALL, mk

pytestmark = pytest.mark.gpu

LAYOUTS = [B.DW_OIHW, B.DW_OHWI, B.DW_HWIO]
assert (B.DW_OIHW, B.DW_OHWI, B.DW_HWIO) == (oracle.OIHW, oracle.OHWI, oracle.HWIO)
CASES = [SMALL[i] for i in (0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 16, 17, 20, 24, 25, 26, 27, 28, 29, 30)]


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("t", CASES)
def test_approx_nhwc_matches_oracle(t, layout, dtype):
    import torch
    d = mk(t, dtype)
    X, dY = rand_inputs(d, 1357, dtype)
    Xl = oracle.x_to_nhwc(X)
    idx = torch.empty((d.N, d.K), dtype=torch.int32, device="cuda")
    S = torch.empty((d.N, d.K), dtype=torch.float32, device="cuda")
    got = B.conv_wgrad_approx_nhwc(d, to_gpu(Xl), to_gpu(dY), layout, scale=0.5, idx_out=idx, sum_out=S).cpu().numpy()
    want, _, _ = oracle.wgrad_approx_nhwc(oracle_shape(d), Xl, dY, 0.5, layout)
    assert got.shape == want.shape
    check_select(d, dY, idx.cpu().numpy(), S.cpu().numpy())
    assert normwise_err(got, want) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("t", [SMALL[i] for i in (0, 1, 2, 5, 7, 8, 9, 11, 18, 20)])
def test_exact_nhwc_matches_oracle(t, layout, dtype):
    d = mk(t, dtype)
    X, dY = rand_inputs(d, 2468, dtype)
    Xl = oracle.x_to_nhwc(X)
    got = B.conv_wgrad_exact_nhwc(d, to_gpu(Xl), to_gpu(dY), layout).cpu().numpy()
    want = oracle.wgrad_exact_nhwc(oracle_shape(d), Xl, dY, layout)
    assert got.shape == want.shape
    assert normwise_err(got, want) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("nchw", [(2, 3, 5, 7), (3, 64, 8, 8), (2, 65, 9, 15), (1, 1, 1, 1), (5, 16, 32, 32),
                                  (2, 130, 3, 70), (4, 512, 2, 2)])
def test_input_transpose_is_byte_exact_both_ways(nchw, dtype):
    N, C, H, W = nchw
    d = B.desc(N, C, H, W, 4, dtype=B.BF16 if dtype == "bf16" else B.F32)
    rng = np.random.default_rng(N * 1000 + C)
    X = rng.standard_normal(nchw).astype(np.float32)
    if dtype == "bf16":
        X = inputs.float32_to_bf16_bits(X)
    Xl = B.conv_wgrad_transpose_x(d, to_gpu(X), True)
    assert tuple(Xl.shape) == (N, H, W, C)
    bits = (lambda t: t.view(dtype=__import__("torch").int16).cpu().numpy().view(np.uint16)) if dtype == "bf16" \
        else (lambda t: t.cpu().numpy())
    assert np.array_equal(bits(Xl), oracle.x_to_nhwc(X))
    back = B.conv_wgrad_transpose_x(d, Xl, False)
    assert np.array_equal(bits(back), X)


@pytest.mark.parametrize("kcrs", [(16, 16, 3, 3), (19, 5, 3, 2), (64, 3, 5, 5), (1, 1, 1, 1), (260, 80, 3, 3)])
def test_filter_gradient_permutations_are_exact(kcrs):
    K, C, R, S = kcrs
    d = B.desc(1, C, 8, 8, K, R=R, S=S)
    rng = np.random.default_rng(K + C)
    dW = rng.standard_normal(kcrs).astype(np.float32)
    for a in LAYOUTS:
        src = oracle.dw_permute(dW, oracle.OIHW, a)
        for b in LAYOUTS:
            got = B.conv_wgrad_permute_dw(d, to_gpu(src), a, b).cpu().numpy()
            assert np.array_equal(got, oracle.dw_permute(src, a, b)), (a, b)


def test_the_paper_route_equals_the_direct_route():
    # NCHW tensors -> transpose X -> channel-last kernel (OHWI) -> transpose dW (HWIO), as the paper runs its
    # kernel inside an NCHW framework, against the NCHW call followed by a permutation of its result
    d = mk(SMALL[3])
    X, dY = rand_inputs(d, 11)
    Xg, dYg = to_gpu(X), to_gpu(dY)
    Xl = B.conv_wgrad_transpose_x(d, Xg, True)
    ohwi = B.conv_wgrad_approx_nhwc(d, Xl, dYg, B.DW_OHWI, scale=1 / 128)
    hwio = B.conv_wgrad_permute_dw(d, ohwi, B.DW_OHWI, B.DW_HWIO).cpu().numpy()
    direct = B.conv_wgrad_approx(d, Xg, dYg, scale=1 / 128).cpu().numpy()
    assert normwise_err(hwio, oracle.dw_permute(direct, oracle.OIHW, oracle.HWIO).astype(np.float64)) <= TOL["fp32"]
    want, _, _ = oracle.wgrad_approx(oracle_shape(d), X, dY, scale=1 / 128)
    assert normwise_err(hwio, oracle.dw_permute(want, oracle.OIHW, oracle.HWIO)) <= TOL["fp32"]


def test_outputs_are_overwritten_and_runs_repeat():
    import torch
    d = mk(SMALL[14])
    X, dY = rand_inputs(d, 3)
    Xl, dYg = to_gpu(oracle.x_to_nhwc(X)), to_gpu(dY)
    dW = torch.full(B.dw_shape(d, B.DW_HWIO), float("nan"), device="cuda")
    a = B.conv_wgrad_approx_nhwc(d, Xl, dYg, B.DW_HWIO, dW=dW).clone()
    b = B.conv_wgrad_approx_nhwc(d, Xl, dYg, B.DW_HWIO, dW=dW).clone()
    assert torch.equal(a, b) and torch.isfinite(a).all()
    dW.fill_(float("nan"))
    c = B.conv_wgrad_exact_nhwc(d, Xl, dYg, B.DW_HWIO, dW=dW).clone()
    e = B.conv_wgrad_exact_nhwc(d, Xl, dYg, B.DW_HWIO, dW=dW).clone()
    assert torch.equal(c, e) and torch.isfinite(c).all()


def test_workload_layers_at_full_size():
    # a shallow and a deep ResNet-20 layer and a wide VGG-19 layer at the benchmark batch
    for layer, N in ((inputs.resnet20_stack()[1], 128), (inputs.resnet20_stack()[-1], 128), (inputs.vgg19_stack()[9], 32)):
        d = B.desc_for(layer, N)
        X, dY = rand_inputs(d, 17)
        Xl = oracle.x_to_nhwc(X)
        got = B.conv_wgrad_approx_nhwc(d, to_gpu(Xl), to_gpu(dY), B.DW_OHWI, scale=1 / 128).cpu().numpy()
        want, _, _ = oracle.wgrad_approx_nhwc(oracle_shape(d), Xl, dY, 1 / 128, oracle.OHWI)
        assert normwise_err(got, want) <= TOL["fp32"], layer.name


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("t", [SMALL[0], SMALL[5], SMALL[9], SMALL[20]])
def test_tensors_that_are_only_element_aligned(t, dtype):
    """X and dY start one element into their allocations: no 16-byte access may be used on them."""
    d = mk(t, dtype)
    X, dY = rand_inputs(d, 78, dtype)
    Xl = oracle.x_to_nhwc(X)

    def shifted(a):
        flat = to_gpu(np.concatenate([a.ravel()[:1], a.ravel()]))
        return flat[1:].view(a.shape)
    Xg, dYg = shifted(Xl), shifted(dY)
    assert Xg.data_ptr() % 16 != 0 and dYg.data_ptr() % 16 != 0
    g = oracle_shape(d)
    got = B.conv_wgrad_approx_nhwc(d, Xg, dYg, B.DW_HWIO).cpu().numpy()
    assert normwise_err(got, oracle.wgrad_approx_nhwc(g, Xl, dY, 1.0, oracle.HWIO)[0]) <= TOL[dtype]
    got = B.conv_wgrad_exact_nhwc(d, Xg, dYg, B.DW_OHWI).cpu().numpy()
    assert normwise_err(got, oracle.wgrad_exact_nhwc(g, Xl, dY, oracle.OHWI)) <= TOL[dtype]
    back = B.conv_wgrad_transpose_x(d, Xg, False)
    assert np.array_equal(back.view(dtype=__import__("torch").int16).cpu().numpy().view(np.uint16) if dtype == "bf16"
                          else back.cpu().numpy(), X)
