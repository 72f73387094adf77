"""GPU parity: every entry point of libwgrad, through the C ABI, element by element
against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

import oracle
from paper_1908_05460_amd import binding as B, inputs
from tests.gpu_util import (TOL, as_float32, check_select, normwise_err, oracle_shape, rand_inputs,
                            to_gpu)

pytestmark = pytest.mark.gpu

# N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w  -- several tiles plus ragged tails
SMALL = [
    (16, 16, 32, 32, 16, 3, 3, 1, 1, 1, 1),     # the small configuration
    (3, 3, 32, 32, 16, 3, 3, 1, 1, 1, 1),       # first layer: C = 3 (flat column mapping)
    (5, 16, 32, 32, 32, 3, 3, 2, 2, 1, 1),      # stride 2
    (9, 32, 16, 16, 32, 3, 3, 1, 1, 1, 1),
    (7, 64, 8, 8, 64, 3, 3, 1, 1, 1, 1),
    (20, 64, 4, 4, 128, 3, 3, 1, 1, 1, 1),      # small planes: several images per tile
    (37, 48, 2, 2, 80, 3, 3, 1, 1, 1, 1),       # 2x2 planes, ragged K and image groups
    (4, 5, 9, 7, 19, 3, 3, 1, 1, 1, 1),         # nothing divisible by anything
    (3, 7, 11, 13, 21, 3, 2, 2, 1, 1, 0),       # non-square filter, mixed stride and padding
    (2, 64, 6, 6, 24, 1, 1, 1, 1, 0, 0),        # 1x1: a plain GEMM
    (2, 70, 6, 6, 24, 1, 1, 1, 1, 0, 0),
    (2, 4, 12, 12, 8, 5, 5, 1, 1, 2, 2),        # 5x5
    (1, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0),          # degenerate: a single multiply
    (2, 2, 3, 40, 3, 3, 3, 1, 1, 1, 1),         # wide and flat
    (130, 16, 8, 8, 16, 3, 3, 1, 1, 1, 1),      # long batch, many reduction splits
    (6, 80, 4, 4, 260, 3, 3, 1, 1, 1, 1),       # many output channels on tiny planes (LDS gather, ragged tiles)
    (5, 32, 8, 8, 64, 3, 3, 2, 2, 1, 1),        # stride 2 on small planes
    (40, 64, 2, 2, 512, 3, 3, 1, 1, 1, 1),      # 2x2 planes: most taps fall on padding
    (6, 16, 32, 32, 64, 3, 3, 1, 1, 1, 1),      # K a multiple of 64: the bf16 matrix-core kernel when the dtype is bf16
    (12, 32, 16, 16, 64, 3, 3, 1, 1, 1, 1),
    (24, 128, 8, 8, 192, 3, 3, 1, 1, 1, 1),     # several K tiles and channel tiles, four images per tile
    (33, 16, 4, 4, 64, 3, 3, 1, 1, 1, 1),       # 4x4 planes, a ragged last image group
    (5, 32, 6, 6, 144, 3, 3, 1, 1, 1, 1),       # 6x6 planes: a 16-byte piece of a plane wraps over rows (LDS gather)
    (9, 70, 2, 6, 130, 3, 3, 1, 1, 1, 1),       # 2x6 planes, ragged channel tile
    (3, 1, 16, 16, 5, 3, 9, 1, 1, 4, 4),        # wide filter (S > 8), padding of several columns
    (2, 2, 20, 20, 4, 17, 3, 1, 1, 8, 1),       # tall filter (R > 16)
    (2, 1, 24, 24, 3, 9, 9, 1, 1, 4, 4),        # 81 taps: more than the fused form's tap mask holds
    (11, 16, 1, 4, 32, 3, 3, 1, 1, 1, 1),       # 1x4 planes: maps of four positions (fp32: exact kernel on the sparsified dY)
    (6, 128, 16, 16, 24, 3, 3, 1, 1, 1, 1),     # 1152 entries per output channel: two slices of the fused form
    (3, 200, 8, 8, 10, 3, 3, 1, 1, 1, 1),       # 1800 entries: four slices, a ragged last one; 8x8 maps
    (5, 70, 12, 12, 7, 5, 5, 1, 1, 2, 2),       # 1750 entries of a 5x5 filter
]


def mk(t, dtype="fp32"):
    N, C, H, W, K, R, S, sh, sw, ph, pw = t
    return B.desc(N, C, H, W, K, R, S, stride=sh, pad=ph, stride_w=sw, pad_w=pw,
                  dtype=B.BF16 if dtype == "bf16" else B.F32)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("t", SMALL)
def test_exact_matches_oracle(t, dtype):
    d = mk(t, dtype)
    X, dY = rand_inputs(d, 1234, dtype)
    got = B.conv_wgrad_exact(d, to_gpu(X), to_gpu(dY)).cpu().numpy()
    want = oracle.wgrad_exact(oracle_shape(d), X, dY)
    assert normwise_err(got, want) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("t", SMALL)
def test_approx_matches_oracle(t, dtype):
    import torch
    d = mk(t, dtype)
    X, dY = rand_inputs(d, 4321, dtype)
    idx = torch.empty((d.N, d.K), dtype=torch.int32, device="cuda")
    S = torch.empty((d.N, d.K), dtype=torch.float32, device="cuda")
    got = B.conv_wgrad_approx(d, to_gpu(X), to_gpu(dY), idx_out=idx, sum_out=S).cpu().numpy()
    want, _, _ = oracle.wgrad_approx(oracle_shape(d), X, dY)
    check_select(d, dY, idx.cpu().numpy(), S.cpu().numpy())
    assert normwise_err(got, want) <= TOL[dtype]


# 3x3, stride 1, padding 1 on planes of 4, 8, 16 and 32 columns with 32 or 64 output channels: the position orders of
# the streaming kernel that leave out the taps which meet only padding (column-uniform; image-uniform on 4x4 planes
# in tiles of eight images), and their neighbours that fall back to the row-major order (batches the tiles do not divide)
SKIP_ORDERS = [
    (16, 32, 4, 4, 64), (8, 16, 4, 4, 128), (12, 16, 4, 4, 64), (6, 16, 4, 4, 64), (5, 16, 4, 4, 64),
    (8, 16, 8, 8, 64), (6, 32, 8, 8, 128), (3, 16, 8, 8, 64),
    (4, 16, 16, 16, 64), (3, 16, 16, 16, 32), (2, 32, 16, 16, 128),
    (2, 16, 32, 32, 64), (3, 16, 32, 32, 64),
]


@pytest.mark.parametrize("t", SKIP_ORDERS)
def test_exact_orders_that_leave_out_padding_taps(t):
    N, C, H, W, K = t
    d = B.desc(N, C, H, W, K, R=3, S=3, pad=1)
    X, dY = rand_inputs(d, 5150 + N + H)
    g = oracle_shape(d)
    want = oracle.wgrad_exact(g, X, dY)
    assert normwise_err(B.conv_wgrad_exact(d, to_gpu(X), to_gpu(dY)).cpu().numpy(), want) <= TOL["fp32"]
    # the same layer beside one of another shape in a schedule run (the multi-shape launch's instantiations)
    import torch
    d2 = B.desc(8, 16, 8, 8, 64, R=3, S=3, pad=1)
    X2, dY2 = rand_inputs(d2, 6160 + N + H)
    dWs = [torch.empty((K, C, 3, 3), device="cuda"), torch.empty((64, 16, 3, 3), device="cuda")]
    S = B.Schedule([d, d2], [to_gpu(X), to_gpu(X2)], [to_gpu(dY), to_gpu(dY2)], dWs)
    mask = np.full(2, B.EXACT, np.uint8)
    S.run(mask, B.alloc_workspace(S.workspace_bytes(mask)))
    torch.cuda.synchronize()
    assert normwise_err(dWs[0].cpu().numpy(), want) <= TOL["fp32"]
    assert normwise_err(dWs[1].cpu().numpy(), oracle.wgrad_exact(oracle_shape(d2), X2, dY2)) <= TOL["fp32"]


# bf16 matrix-core kernel with a last tile of fewer than sixteen input channels (the missing ones stay zero in LDS)
RAGGED_C = [(4, 3, 32, 32, 64), (6, 20, 16, 16, 64), (8, 35, 8, 8, 128), (16, 17, 4, 4, 64), (16, 40, 2, 2, 64), (3, 1, 16, 16, 64)]


@pytest.mark.parametrize("t", RAGGED_C)
def test_bf16_matrix_core_kernel_with_a_ragged_channel_tile(t):
    N, C, H, W, K = t
    d = B.desc(N, C, H, W, K, R=3, S=3, pad=1, dtype=B.BF16)
    X, dY = rand_inputs(d, 8800 + C, "bf16")
    g = oracle_shape(d)
    got = B.conv_wgrad_exact(d, to_gpu(X), to_gpu(dY)).cpu().numpy()
    assert normwise_err(got, oracle.wgrad_exact(g, X, dY)) <= TOL["bf16"]
    got = B.conv_wgrad_approx(d, to_gpu(X), to_gpu(dY)).cpu().numpy()
    assert normwise_err(got, oracle.wgrad_approx(g, X, dY)[0]) <= TOL["bf16"]


def test_strided_input_whose_planes_exceed_the_fused_offset_field():
    """70 channels of 512x512 under stride 16: maps of 1024 positions and 70 entries per output channel, the
    shape class of the fused form, but tap offsets inside one image need more than 24 bits."""
    d = mk((2, 70, 512, 512, 4, 1, 1, 16, 16, 0, 0))
    X, dY = rand_inputs(d, 99)
    Xg, dYg = to_gpu(X), to_gpu(dY)
    g = oracle_shape(d)
    assert normwise_err(B.conv_wgrad_approx(d, Xg, dYg).cpu().numpy(), oracle.wgrad_approx(g, X, dY)[0]) <= TOL["fp32"]
    assert normwise_err(B.conv_wgrad_approx_topk(d, Xg, dYg, 3).cpu().numpy(),
                        oracle.wgrad_approx_topk(g, X, dY, 3)[0]) <= TOL["fp32"]
    assert normwise_err(B.conv_wgrad_exact(d, Xg, dYg).cpu().numpy(), oracle.wgrad_exact(g, X, dY)) <= TOL["fp32"]


# shapes whose output rows are too wide (or whose strides spread them too far) for a tile of whole rows in
# LDS: the general form of the exact kernel
WIDE = [
    (2, 5, 6, 1024, 7, 3, 3, 1, 1, 1, 1),       # wide and flat
    (1, 3, 40, 300, 70, 3, 7, 1, 1, 1, 3),      # ragged everything, 63 entries per output channel
    (2, 16, 4, 1024, 20, 1, 9, 1, 1, 0, 4),     # a 1-d convolution
    (3, 70, 9, 640, 130, 2, 2, 3, 16, 1, 0),    # stride 16 along a wide row: ragged tiles both ways
    (2, 64, 12, 512, 64, 3, 3, 1, 1, 1, 1),     # the matrix-core kernels' favourite filter on rows of 512
]


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("t", WIDE)
def test_exact_general_form_matches_oracle(t, dtype):
    d = mk(t, dtype)
    X, dY = rand_inputs(d, 777, dtype)
    g = oracle_shape(d)
    want = oracle.wgrad_exact(g, X, dY)
    got = B.conv_wgrad_exact(d, to_gpu(X), to_gpu(dY)).cpu().numpy()
    assert normwise_err(got, want) <= TOL[dtype]
    # the same through the channel-last entry point and through a schedule of two such layers
    got = B.conv_wgrad_exact_nhwc(d, to_gpu(oracle.x_to_nhwc(X)), to_gpu(dY), B.DW_OIHW).cpu().numpy()
    assert normwise_err(got, want) <= TOL[dtype]
    import torch
    Xg, dYg = to_gpu(X), to_gpu(dY)
    dWs = [torch.full((d.K, d.C, d.R, d.S), float("nan"), device="cuda") for _ in range(2)]
    sch = B.Schedule([d, d], [Xg, Xg], [dYg, dYg], dWs)
    m = [B.EXACT, B.EXACT]
    sch.run(m, B.alloc_workspace(sch.workspace_bytes(m), "cuda"))
    for dW in dWs:
        assert normwise_err(dW.cpu().numpy(), want) <= TOL[dtype]


def test_approx_scale_is_applied_once_and_power_of_two_is_bit_exact():
    d = mk(SMALL[0])
    X, dY = rand_inputs(d, 5)
    Xg, dYg = to_gpu(X), to_gpu(dY)
    one = B.conv_wgrad_approx(d, Xg, dYg, scale=1.0).cpu().numpy()
    scaled = B.conv_wgrad_approx(d, Xg, dYg, scale=1 / 128).cpu().numpy()
    assert np.array_equal(scaled, one * np.float32(1 / 128))
    want, _, _ = oracle.wgrad_approx(oracle_shape(d), X, dY, scale=1 / 128)
    assert normwise_err(scaled, want) <= TOL["fp32"]


def test_outputs_are_overwritten_not_accumulated_and_runs_are_deterministic():
    import torch
    d = mk(SMALL[3])
    X, dY = rand_inputs(d, 6)
    Xg, dYg = to_gpu(X), to_gpu(dY)
    dW = torch.full((d.K, d.C, d.R, d.S), 7.0, device="cuda")
    a = B.conv_wgrad_exact(d, Xg, dYg, dW=dW).clone()
    b = B.conv_wgrad_exact(d, Xg, dYg, dW=dW).clone()
    assert torch.equal(a, b)
    dW.fill_(float("nan"))
    c = B.conv_wgrad_approx(d, Xg, dYg, dW=dW).clone()
    e = B.conv_wgrad_approx(d, Xg, dYg, dW=dW).clone()
    assert torch.equal(c, e) and torch.isfinite(c).all()


def test_zero_dY_gives_exact_zero_and_one_hot_maps_make_approx_equal_exact():
    import torch
    d = mk(SMALL[2])
    X, dY = rand_inputs(d, 7)
    Xg = to_gpu(X)
    z = torch.zeros((d.N, d.K, d.Ho, d.Wo), device="cuda")
    assert not B.conv_wgrad_exact(d, Xg, z).any() and not B.conv_wgrad_approx(d, Xg, z).any()
    rng = np.random.default_rng(8)
    one = np.zeros((d.N, d.K, d.Ho * d.Wo), np.float32)
    pos = rng.integers(0, d.Ho * d.Wo, size=(d.N, d.K))
    np.put_along_axis(one, pos[..., None], rng.standard_normal((d.N, d.K, 1)).astype(np.float32), axis=2)
    og = to_gpu(one.reshape(d.N, d.K, d.Ho, d.Wo))
    ex = B.conv_wgrad_exact(d, Xg, og).cpu().numpy()
    ap = B.conv_wgrad_approx(d, Xg, og).cpu().numpy()
    assert normwise_err(ap, ex.astype(np.float64)) <= 1e-5


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("t", [SMALL[0], SMALL[5], SMALL[9]])
def test_tensors_that_are_only_element_aligned(t, dtype):
    """X and dY start one element into their allocations: the 16-byte paths must not be taken."""
    import torch
    d = mk(t, dtype)
    X, dY = rand_inputs(d, 77, dtype)

    def shifted(a):
        flat = to_gpu(np.concatenate([a.ravel()[:1], a.ravel()]))
        return flat[1:].view(a.shape)
    Xg, dYg = shifted(X), shifted(dY)
    assert Xg.data_ptr() % 16 != 0 and Xg.is_contiguous()
    g = oracle_shape(d)
    assert normwise_err(B.conv_wgrad_exact(d, Xg, dYg).cpu().numpy(), oracle.wgrad_exact(g, X, dY)) <= TOL[dtype]
    idx = torch.empty((d.N, d.K), dtype=torch.int32, device="cuda")
    S = torch.empty((d.N, d.K), dtype=torch.float32, device="cuda")
    got = B.conv_wgrad_approx(d, Xg, dYg, idx_out=idx, sum_out=S).cpu().numpy()
    check_select(d, dY, idx.cpu().numpy(), S.cpu().numpy())
    assert normwise_err(got, oracle.wgrad_approx(g, X, dY)[0]) <= TOL[dtype]


# ---- selection: ties and degenerate maps, bit-exact -------------------------------------

@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("hw", [(1, 1), (2, 2), (1, 3), (4, 4), (3, 5), (8, 8), (7, 9), (16, 16), (32, 32), (33, 31), (64, 48)])
def test_select_with_heavy_ties(hw, dtype):
    Ho, Wo = hw
    d = B.desc(6, 1, Ho, Wo, 11, R=1, S=1, pad=0, dtype=B.BF16 if dtype == "bf16" else B.F32)
    rng = np.random.default_rng(Ho * 100 + Wo)
    dY = (rng.integers(-3, 4, size=(d.N, d.K, Ho, Wo)) * 0.25).astype(np.float32)   # few distinct magnitudes
    dY[0, 0] = 0.0                                   # all-zero map -> position 0
    dY[0, 1] = 0.0; dY[0, 1].flat[-1] = -1e-20       # single tiny value in the last position
    dY[0, 2] = -0.0
    if dtype == "bf16":
        dY = inputs.float32_to_bf16_bits(dY)
    idx, S = B.conv_wgrad_select(d, to_gpu(dY))
    check_select(d, dY, idx.cpu().numpy(), S.cpu().numpy())


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("hw", [(2, 2), (4, 4), (8, 8), (16, 16), (32, 32), (7, 9)])
def test_select_ranks_nan_as_zero(hw, dtype):
    """A NaN ranks as a zero of its map (lowest position among equal magnitudes wins): positions bit-exact
    against the oracle through the selection call, the approximation call (fused / LDS / sparsified forms)
    and the top-k call; sums of maps that hold a NaN are NaN on both sides and are not compared."""
    import torch
    Ho, Wo = hw
    d = B.desc(8, 16, Ho, Wo, 16, R=3, S=3, pad=1, dtype=B.BF16 if dtype == "bf16" else B.F32)
    rng = np.random.default_rng(Ho * 37 + Wo)
    dY = (rng.integers(-2, 3, size=(d.N, d.K, Ho, Wo)) * 0.5).astype(np.float32)
    L = Ho * Wo
    dY[0, 0] = 0.0; dY[0, 0].flat[0] = np.nan                       # NaN at position 0, zeros elsewhere
    dY[0, 1] = 0.0; dY[0, 1].flat[L - 1] = np.nan                   # zeros, then a NaN at the end
    dY[0, 2] = np.nan                                               # only NaNs
    dY[0, 3] = 0.0; dY[0, 3].flat[0] = np.nan; dY[0, 3].flat[L - 1] = 1e-20   # a tiny value beats the NaN
    dY[1, 0].flat[rng.integers(0, L, 3)] = -np.nan                  # NaNs inside an ordinary map
    X = np.maximum(rng.standard_normal((d.N, d.C, Ho, Wo)).astype(np.float32), 0)
    if dtype == "bf16":
        dY, X = inputs.float32_to_bf16_bits(dY), inputs.float32_to_bf16_bits(X)
    want_idx, _ = oracle.select(oracle_shape(d), dY)
    assert want_idx[0, :4].tolist() == [0, 0, 0, L - 1]
    idx, _ = B.conv_wgrad_select(d, to_gpu(dY))
    assert np.array_equal(idx.cpu().numpy(), want_idx)
    idx2 = torch.empty((d.N, d.K), dtype=torch.int32, device="cuda")
    B.conv_wgrad_approx(d, to_gpu(X), to_gpu(dY), idx_out=idx2)
    assert np.array_equal(idx2.cpu().numpy(), want_idx)
    k = min(3, L)
    idx3 = torch.empty((d.N, d.K, k), dtype=torch.int32, device="cuda")
    B.conv_wgrad_approx_topk(d, to_gpu(X), to_gpu(dY), k, idx_out=idx3)
    assert np.array_equal(idx3.cpu().numpy(), oracle.select_topk(oracle_shape(d), dY, k)[0])


def test_select_on_workload_gradients_fp32_and_bf16():
    for dtype in ("fp32", "bf16"):
        d = B.desc(32, 1, 32, 32, 64, R=1, S=1, pad=0, dtype=B.BF16 if dtype == "bf16" else B.F32)
        _, dY = rand_inputs(d, 99, dtype)
        idx, S = B.conv_wgrad_select(d, to_gpu(dY))
        check_select(d, dY, idx.cpu().numpy(), S.cpu().numpy())


# ---- trivial methods -------------------------------------------------------------------

def test_zero_gradient():
    import torch
    d = mk(SMALL[7])
    dW = torch.full((d.K, d.C, d.R, d.S), 3.0, device="cuda")
    B.conv_wgrad_zero(d, dW)
    assert not dW.any()


def test_random_gradient_small_radii_are_accurate():
    """19 million draws: a few of them have u1 within 1e-6 of 1, where the radius sqrt(-2 ln u1) is small and a
    uniform that was rounded to fp32 would cost it several digits.  Absolute and relative accuracy of every value."""
    import torch
    d = B.desc(1, 1024, 8, 8, 2048)
    n = d.K * d.C * 9
    sigma, seed, offset = 1 / 128, 20190814, 3
    dW = torch.empty((d.K, d.C, 3, 3), device="cuda")
    B.conv_wgrad_random(d, dW, sigma, seed, offset)
    got = dW.cpu().numpy().ravel().astype(np.float64)
    want = oracle.random_normal(seed, offset, n, sigma)
    assert np.abs(got - want).max() <= 2e-6 * sigma
    big = np.abs(want) > 1e-4 * sigma
    assert (np.abs(got - want)[big] / np.abs(want)[big]).max() <= 1e-4


def test_random_gradient_matches_oracle_stream_value_by_value():
    import torch
    d = B.desc(1, 64, 8, 8, 129)                      # 74304 values
    n = d.K * d.C * 9
    sigma, seed = 1 / 128, 190805460
    # four stream positions share a generator call: offsets in every residue mod 4, and across the 2^32 counter boundary
    for offset in (0, 12345, 2, 7, (1 << 32) - 1000, (1 << 34) - 1001):
        dW = torch.empty((d.K, d.C, 3, 3), device="cuda")
        B.conv_wgrad_random(d, dW, sigma, seed, offset)
        want = oracle.random_normal(seed, offset, n, sigma)
        got = dW.cpu().numpy().ravel().astype(np.float64)
        assert np.abs(got - want).max() <= 2e-5 * sigma          # fp32 log/sqrt/sin/cos vs fp64
    # tensors smaller than a call, and a tensor that is only element-aligned, with a guard element on either side
    for (K, C), offset in (((1, 1), 3), ((1, 1), 0), ((2, 1), 1), ((7, 3), 6)):
        t = B.desc(1, C, 8, 8, K)
        m = K * C * 9
        buf = torch.full((m + 2,), 7.0, device="cuda")
        B.conv_wgrad_random(t, buf[1:m + 1].view(K, C, 3, 3), sigma, seed, offset)
        got = buf.cpu().numpy().astype(np.float64)
        assert got[0] == 7.0 and got[-1] == 7.0
        assert np.abs(got[1:-1] - oracle.random_normal(seed, offset, m, sigma)).max() <= 2e-5 * sigma
    a = torch.empty((d.K, d.C, 3, 3), device="cuda"); b = torch.empty_like(a)
    B.conv_wgrad_random(d, a, sigma, seed, 0); B.conv_wgrad_random(d, b, sigma, seed, n)
    assert not torch.equal(a, b)                      # a new batch (advanced offset) draws new numbers
    z = a.cpu().numpy().ravel() / sigma
    assert abs(z.mean()) < 4 / np.sqrt(n) and abs(z.std() - 1) < 0.02


def test_schedule_run_equals_the_individual_calls():
    import torch
    from paper_1908_05460_amd import schedule as sch
    stack, N = inputs.resnet20_stack(), 4
    descs = [B.desc_for(l, N) for l in stack]
    data = [inputs.make_layer_inputs(l, N, config=2, layer_index=i) for i, l in enumerate(stack)]
    Xs = [to_gpu(x) for x, _ in data]; dYs = [to_gpu(y) for _, y in data]
    dWs = [torch.empty((l.K, l.C, 3, 3), device="cuda") for l in stack]
    s = B.Schedule(descs, Xs, dYs, dWs)
    methods = sch.every_other_layer(len(stack), 0)
    methods[4] = sch.ZERO; methods[6] = sch.RANDOM
    ws = B.alloc_workspace(s.workspace_bytes(methods))
    s.run(methods, ws, scale=0.5, sigma=1 / 128, seed=3, offset=1000)
    off = 1000
    for i, l in enumerate(stack):
        ref = torch.empty_like(dWs[i])
        if methods[i] == sch.EXACT: B.conv_wgrad_exact(descs[i], Xs[i], dYs[i], dW=ref)
        elif methods[i] == sch.APPROX: B.conv_wgrad_approx(descs[i], Xs[i], dYs[i], scale=0.5, dW=ref)
        elif methods[i] == sch.ZERO: B.conv_wgrad_zero(descs[i], ref)
        else: B.conv_wgrad_random(descs[i], ref, 1 / 128, 3, off)
        assert torch.equal(ref, dWs[i]), l.name
        off += ref.numel()


def test_exact_schedule_with_more_groups_and_layers_than_one_multi_shape_launch_carries():
    """Thirty exact fp32 layers of ten shapes that the multi-shape launch takes: more than nine groups and more
    than 24 layers, so the launch is issued in parts; every layer against its individual call."""
    import torch
    shapes = [(16, 32, 16), (16, 16, 32), (32, 16, 32), (64, 8, 64), (3, 32, 64), (64, 32, 64), (64, 16, 128),
              (64, 4, 64), (32, 2, 32), (16, 2, 16)]                       # (C, H = W, K)
    N, per_shape = 8, 3
    descs, Xs, dYs, dWs = [], [], [], []
    for rep in range(per_shape):
        for i, (C, HW, K) in enumerate(shapes):
            d = B.desc(N, C, HW, HW, K, R=3, S=3, pad=1)
            X, dY = rand_inputs(d, 7000 + 10 * rep + i)
            descs.append(d); Xs.append(to_gpu(X)); dYs.append(to_gpu(dY))
            dWs.append(torch.full((K, C, 3, 3), float("nan"), device="cuda"))
    s = B.Schedule(descs, Xs, dYs, dWs)
    mask = np.full(len(descs), B.EXACT, np.uint8)
    s.run(mask, B.alloc_workspace(s.workspace_bytes(mask)))
    torch.cuda.synchronize()
    for d, X, dY, dW in zip(descs, Xs, dYs, dWs):
        ref = B.conv_wgrad_exact(d, X, dY)
        assert normwise_err(dW.cpu().numpy(), ref.cpu().numpy().astype(np.float64)) <= 1e-5


def test_schedule_run_with_more_layers_than_one_table_or_group_holds():
    """70 layers of five shapes and two dtypes, all four methods: groups of identical layers overflow
    (more than 8 per shape and method) and so do the tables of the reduction and of the fills (more
    than 32 tensors); every layer must still get the result of its individual call."""
    import torch
    from paper_1908_05460_amd import schedule as sch
    shapes = [SMALL[0], SMALL[3], SMALL[4], SMALL[5], SMALL[18]]
    nl = 70
    descs, Xs, dYs, dWs, methods = [], [], [], [], []
    for i in range(nl):
        dtype = "bf16" if i % 7 == 3 else "fp32"
        d = mk(shapes[i % len(shapes)], dtype)
        X, dY = rand_inputs(d, 100 + i, dtype)
        descs.append(d); Xs.append(to_gpu(X)); dYs.append(to_gpu(dY))
        dWs.append(torch.full((d.K, d.C, d.R, d.S), float("nan"), device="cuda"))
        methods.append([sch.EXACT, sch.APPROX, sch.EXACT, sch.ZERO, sch.APPROX, sch.RANDOM][i % 6])
    methods = np.array(methods, np.uint8)
    s = B.Schedule(descs, Xs, dYs, dWs)
    ws = B.alloc_workspace(s.workspace_bytes(methods))
    s.run(methods, ws, scale=0.25, sigma=1 / 128, seed=11, offset=5)
    off = 5
    for i in range(nl):
        ref = torch.empty_like(dWs[i])
        if methods[i] == sch.EXACT: B.conv_wgrad_exact(descs[i], Xs[i], dYs[i], dW=ref)
        elif methods[i] == sch.APPROX: B.conv_wgrad_approx(descs[i], Xs[i], dYs[i], scale=0.25, dW=ref)
        elif methods[i] == sch.ZERO: B.conv_wgrad_zero(descs[i], ref)
        else: B.conv_wgrad_random(descs[i], ref, 1 / 128, 11, off)
        if methods[i] in (sch.ZERO, sch.RANDOM):
            assert torch.equal(ref, dWs[i]), i
        else:   # the folded launch may split the reduction differently: same sum, another order
            err = (ref - dWs[i]).abs().max().item() / max(ref.abs().max().item(), 1e-30)
            assert err < 1e-5, (i, err)
        off += ref.numel()
