"""GPU parity of the top-k form of the approximation (Section 2.3), through the C ABI:
kept positions bit-exact and in rank order, sums and filter gradient within tolerance."""
import numpy as np
import pytest

import oracle
from paper_1908_05460_amd import binding as B, inputs
from tests.gpu_util import S_TOL, TOL, as_float32, normwise_err, oracle_shape, rand_inputs, to_gpu
from tests.test_gpu_parity import SMALL, mk

pytestmark = pytest.mark.gpu


def run(d, X, dY, k, scale=1.0):
    import torch
    idx = torch.full((d.N, d.K, k), -7, dtype=torch.int32, device="cuda")
    S = torch.empty((d.N, d.K), dtype=torch.float32, device="cuda")
    dW = B.conv_wgrad_approx_topk(d, to_gpu(X), to_gpu(dY), k, scale=scale, idx_out=idx, sum_out=S)
    return dW.cpu().numpy(), idx.cpu().numpy(), S.cpu().numpy()


def check(d, X, dY, k, dtype, scale=1.0):
    got, idx, S = run(d, X, dY, k, scale)
    want, want_idx, want_S = oracle.wgrad_approx_topk(oracle_shape(d), X, dY, k, scale)
    assert np.array_equal(idx, want_idx), "kept positions differ from the oracle"
    bound = S_TOL * np.abs(as_float32(dY).astype(np.float64)).reshape(d.N, d.K, -1).sum(axis=2)
    assert np.all(np.abs(S.astype(np.float64) - want_S) <= bound + 1e-30)
    assert normwise_err(got, want) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("k", [1, 2, 3, 4, 8])
@pytest.mark.parametrize("t", [SMALL[i] for i in (0, 1, 2, 4, 5, 6, 7, 8, 11, 13, 14, 15, 17, 20, 24, 25, 26, 27, 28, 29, 30)])
def test_topk_matches_oracle(t, k, dtype):
    d = mk(t, dtype)
    if k > d.Ho * d.Wo:
        assert B.topk_workspace_bytes(d, k) == 0
        pytest.skip("k exceeds the map")
    X, dY = rand_inputs(d, 2468 + k, dtype)
    check(d, X, dY, k, dtype)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("hw,k", [((1, 1), 1), ((2, 2), 4), ((1, 3), 2), ((4, 4), 16), ((8, 8), 5), ((7, 9), 63),
                                  ((16, 16), 7), ((17, 16), 9), ((32, 32), 64), ((33, 31), 12), ((64, 48), 6),
                                  ((41, 25), 4), ((64, 64), 3), ((80, 64), 5), ((3, 1700), 8)])
def test_topk_order_under_heavy_ties(hw, k, dtype):
    # few distinct magnitudes: the order among equals (lower flat index first) decides nearly every rank;
    # the map lengths cover every register-resident variant of the selection (a wavefront per map up to 1024
    # positions, a workgroup per map beyond) and the re-reading one (more than 4096 positions)
    Ho, Wo = hw
    d = B.desc(5, 2, Ho, Wo, 9, R=1, S=1, pad=0, dtype=B.BF16 if dtype == "bf16" else B.F32)
    rng = np.random.default_rng(Ho * 100 + Wo + k)
    dY = (rng.integers(-3, 4, size=(d.N, d.K, Ho, Wo)) * 0.25).astype(np.float32)
    dY[0, 0] = 0.0                                   # all-zero map: positions 0..k-1
    dY[0, 1] = 0.0; dY[0, 1].flat[-1] = -1e-20       # one tiny value at the end ranks first
    dY[0, 2] = -0.0
    X = rng.standard_normal((d.N, d.C, Ho, Wo)).astype(np.float32)
    if dtype == "bf16":
        dY, X = inputs.float32_to_bf16_bits(dY), inputs.float32_to_bf16_bits(X)
    check(d, X, dY, k, dtype)
    _, idx, _ = run(d, X, dY, k)
    assert np.array_equal(idx[0, 0], np.arange(k)) and idx[0, 1, 0] == Ho * Wo - 1


def test_k_equal_one_is_algorithm_1():
    import torch
    for t in (SMALL[0], SMALL[4], SMALL[7]):
        d = mk(t)
        X, dY = rand_inputs(d, 77)
        got, idx, S = run(d, X, dY, 1)
        idx1 = torch.empty((d.N, d.K), dtype=torch.int32, device="cuda")
        one = B.conv_wgrad_approx(d, to_gpu(X), to_gpu(dY), idx_out=idx1).cpu().numpy()
        assert np.array_equal(idx[:, :, 0], idx1.cpu().numpy())
        assert normwise_err(got, one.astype(np.float64)) <= TOL["fp32"]


def test_k_sparse_maps_give_the_exact_gradient_when_the_kept_values_are_equal():
    # maps whose only nonzeros are k equal values: sum/k is that value, so top-k reproduces the exact gradient
    d = mk(SMALL[3])
    k = 3
    rng = np.random.default_rng(5)
    X = rng.standard_normal((d.N, d.C, d.H, d.W)).astype(np.float32)
    dY = np.zeros((d.N, d.K, d.Ho, d.Wo), np.float32)
    for n in range(d.N):
        for ko in range(d.K):
            pos = rng.choice(d.Ho * d.Wo, size=k, replace=False)
            dY[n, ko].flat[pos] = rng.choice([-0.5, 0.25, 2.0])
    got, _, _ = run(d, X, dY, k)
    exact = B.conv_wgrad_exact(d, to_gpu(X), to_gpu(dY)).cpu().numpy()
    assert normwise_err(got, exact.astype(np.float64)) <= TOL["fp32"]
    assert normwise_err(got, oracle.wgrad_exact(oracle_shape(d), X, dY)) <= TOL["fp32"]


def test_scale_and_overwrite_and_determinism():
    import torch
    d = mk(SMALL[14])
    X, dY = rand_inputs(d, 9)
    Xg, dYg = to_gpu(X), to_gpu(dY)
    dW = torch.full((d.K, d.C, d.R, d.S), float("nan"), device="cuda")
    a = B.conv_wgrad_approx_topk(d, Xg, dYg, 4, dW=dW).clone()
    b = B.conv_wgrad_approx_topk(d, Xg, dYg, 4, dW=dW).clone()
    assert torch.equal(a, b) and torch.isfinite(a).all()
    c = B.conv_wgrad_approx_topk(d, Xg, dYg, 4, scale=1 / 128).cpu().numpy()
    assert np.array_equal(c, a.cpu().numpy() * np.float32(1 / 128))


def test_limits_are_refused_without_a_launch():
    d = mk(SMALL[0])
    X, dY = rand_inputs(d, 1)
    for k in (0, -1, 65, d.Ho * d.Wo + 1):
        assert B.topk_workspace_bytes(d, k) == 0
        with pytest.raises(B.WgradError) as e:
            B.conv_wgrad_approx_topk(d, to_gpu(X), to_gpu(dY), k, ws=B.alloc_workspace(1 << 20))
        assert e.value.status == B.UNSUPPORTED
    need = B.topk_workspace_bytes(d, 4)
    assert need > 0 and need % 256 == 0
    with pytest.raises(B.WgradError) as e:
        B.conv_wgrad_approx_topk(d, to_gpu(X), to_gpu(dY), 4, ws=B.alloc_workspace(need - 256))
    assert e.value.status == B.WORKSPACE_TOO_SMALL


def test_topk_on_a_workload_layer_at_full_size():
    # one deep ResNet-20 layer at the benchmark batch
    layer = inputs.resnet20_stack()[-1]
    d = B.desc_for(layer, 128)
    X, dY = rand_inputs(d, 31)
    check(d, X, dY, 4, "fp32", scale=1 / 128)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("t", [SMALL[0], SMALL[5], SMALL[9], SMALL[20]])
def test_tensors_that_are_only_element_aligned(t, dtype):
    """X and dY start one element into their allocations: the fused and LDS forms must step aside or cope."""
    import torch
    d = mk(t, dtype)
    X, dY = rand_inputs(d, 79, dtype)

    def shifted(a):
        flat = to_gpu(np.concatenate([a.ravel()[:1], a.ravel()]))
        return flat[1:].view(a.shape)
    Xg, dYg = shifted(X), shifted(dY)
    assert Xg.data_ptr() % 16 != 0 and dYg.data_ptr() % 16 != 0
    k = min(3, d.Ho * d.Wo)
    idx = torch.empty((d.N, d.K, k), dtype=torch.int32, device="cuda")
    got = B.conv_wgrad_approx_topk(d, Xg, dYg, k, idx_out=idx).cpu().numpy()
    want, want_idx, _ = oracle.wgrad_approx_topk(oracle_shape(d), X, dY, k)
    assert np.array_equal(idx.cpu().numpy(), want_idx)
    assert normwise_err(got, want) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("k", [1, 3, 8])
def test_topk_through_a_schedule_run(k, dtype):
    """A mixed schedule whose approximated layers take the top-k form: every layer against the oracle; maps
    shorter than k keep all their positions."""
    import torch
    from paper_1908_05460_amd import schedule as sch
    N = 6
    stack = [(3, 32, 16, 1), (16, 32, 16, 1), (16, 32, 16, 1), (16, 16, 32, 2), (32, 8, 64, 1), (64, 4, 128, 1),
             (64, 4, 128, 1), (64, 2, 128, 1), (64, 2, 128, 1)]
    descs = [B.desc(N, C, H, H, K, stride=st, dtype=B.BF16 if dtype == "bf16" else B.F32) for C, H, K, st in stack]
    data = [rand_inputs(d, 70 + i, dtype) for i, d in enumerate(descs)]
    dWs = [torch.full((d.K, d.C, 3, 3), float("nan"), device="cuda") for d in descs]
    s = B.Schedule(descs, [to_gpu(x) for x, _ in data], [to_gpu(y) for _, y in data], dWs)
    # two masks: a mixed one, and one whose repeated shapes are all approximated (those that the fused form takes run
    # as one group of the multi-group launch, the others layer by layer)
    for methods in (np.array([sch.APPROX, sch.EXACT, sch.APPROX, sch.APPROX, sch.APPROX, sch.ZERO, sch.APPROX, sch.APPROX,
                              sch.EXACT], np.uint8),
                    np.array([sch.APPROX] * 8 + [sch.EXACT], np.uint8)):
        for t in dWs:
            t.fill_(float("nan"))
        check_topk_schedule(s, methods, k, descs, data, dWs, stack, dtype)


def check_topk_schedule(s, methods, k, descs, data, dWs, stack, dtype):
    from paper_1908_05460_amd import schedule as sch
    ws = B.alloc_workspace(s.workspace_bytes_topk(methods, k))
    s.run_topk(methods, k, ws, scale=0.5)
    for i, d in enumerate(descs):
        got = dWs[i].cpu().numpy()
        g = oracle_shape(d)
        if methods[i] == sch.EXACT:
            want = oracle.wgrad_exact(g, *data[i])
        elif methods[i] == sch.APPROX:
            want = oracle.wgrad_approx_topk(g, *data[i], min(k, d.Ho * d.Wo), scale=0.5)[0]
        else:
            assert not got.any()
            continue
        assert normwise_err(got, want) <= TOL[dtype], (i, stack[i])
