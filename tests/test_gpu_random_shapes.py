"""Seeded random convolution shapes through every entry point, against the oracle: selected positions
bit-exact, gradients within tolerance.  Two distributions: moderate shapes (filters 1..5, strides 1..3,
padding below the filter size), and extreme ones (filters to 9x11, strides to 7, padding beyond the filter
size, rows of up to 512 elements, single-channel and single-image cases)."""
import numpy as np
import pytest

import oracle
from paper_1908_05460_amd import binding as B
from tests.gpu_util import TOL, check_select, normwise_err, oracle_shape, rand_inputs, to_gpu

pytestmark = pytest.mark.gpu


def moderate(rng):
    R = int(rng.choice([1, 2, 3, 3, 3, 5])); S = int(rng.choice([1, 2, 3, 3, 3, 4]))
    sh = int(rng.choice([1, 1, 1, 2, 3])); sw = int(rng.choice([1, 1, 1, 2]))
    ph = int(rng.integers(0, R)); pw = int(rng.integers(0, S))
    H = int(rng.integers(max(1, R - 2 * ph), 20)); W = int(rng.integers(max(1, S - 2 * pw), 20))
    if rng.random() < 0.3:
        H = W = int(rng.choice([2, 4, 6, 8, 16]))
    C = int(rng.choice([1, 3, 5, 16, 24, 32, 48, 64, 80, 128]))
    K = int(rng.choice([1, 7, 16, 32, 64, 96, 128, 144, 256]))
    N = int(rng.integers(1, 40))
    return N, C, H, W, K, R, S, sh, sw, ph, pw


def extreme(rng):
    R = int(rng.choice([1, 2, 3, 3, 4, 5, 7, 9])); S = int(rng.choice([1, 2, 3, 3, 4, 6, 8, 11]))
    sh = int(rng.choice([1, 1, 2, 3, 5])); sw = int(rng.choice([1, 1, 2, 4, 7]))
    ph = int(rng.integers(0, R + 3)); pw = int(rng.integers(0, S + 3))
    H = int(rng.integers(1, 40)); W = int(rng.integers(1, 40))
    mode = rng.random()
    if mode < 0.2:
        W = int(rng.choice([64, 128, 224, 300, 512])); H = int(rng.integers(1, 6))
    elif mode < 0.3:
        H = int(rng.choice([64, 100, 256])); W = int(rng.integers(1, 6))
    elif mode < 0.4:
        H = W = int(rng.choice([32, 56, 64]))
    C = int(rng.choice([1, 2, 3, 5, 16, 17, 32, 64, 70, 128]))
    K = int(rng.choice([1, 2, 7, 16, 33, 64, 100, 128, 192, 260]))
    N = int(rng.choice([1, 2, 3, 5, 8, 17, 32]))
    return N, C, H, W, K, R, S, sh, sw, ph, pw


def random_cases(seed, count, draw=moderate):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        N, C, H, W, K, R, S, sh, sw, ph, pw = draw(rng)
        dtype = "bf16" if rng.random() < 0.4 else "fp32"
        k = int(rng.integers(1, 6)); layout = int(rng.integers(0, 3))
        if H + 2 * ph < R or W + 2 * pw < S:
            continue
        Ho, Wo = (H + 2 * ph - R) // sh + 1, (W + 2 * pw - S) // sw + 1
        if N * K * Ho * Wo * C * R * S > 2e8 or N * C * H * W > 4e6 or K * C * R * S > 2e6:
            continue
        out.append(pytest.param((N, C, H, W, K, R, S, sh, sw, ph, pw), dtype, min(k, Ho * Wo), layout,
                                id=f"N{N}C{C}H{H}W{W}K{K}R{R}S{S}s{sh}{sw}p{ph}{pw}-{dtype}"))
    return out


@pytest.mark.parametrize("t,dtype,k,layout", random_cases(20190805, 48) + random_cases(1908, 64, extreme))
def test_every_entry_point_on_a_random_shape(t, dtype, k, layout):
    import torch
    N, C, H, W, K, R, S, sh, sw, ph, pw = t
    d = B.desc(N, C, H, W, K, R=R, S=S, stride=sh, pad=ph, stride_w=sw, pad_w=pw, dtype=B.BF16 if dtype == "bf16" else B.F32)
    X, dY = rand_inputs(d, N * 1000 + K, dtype)
    g = oracle_shape(d)
    Xg, dYg = to_gpu(X), to_gpu(dY)
    assert normwise_err(B.conv_wgrad_exact(d, Xg, dYg).cpu().numpy(), oracle.wgrad_exact(g, X, dY)) <= TOL[dtype]
    idx = torch.empty((d.N, d.K), dtype=torch.int32, device="cuda")
    sums = torch.empty((d.N, d.K), dtype=torch.float32, device="cuda")
    got = B.conv_wgrad_approx(d, Xg, dYg, scale=0.5, idx_out=idx, sum_out=sums).cpu().numpy()
    check_select(d, dY, idx.cpu().numpy(), sums.cpu().numpy())
    assert normwise_err(got, oracle.wgrad_approx(g, X, dY, scale=0.5)[0]) <= TOL[dtype]
    idk = torch.empty((d.N, d.K, k), dtype=torch.int32, device="cuda")
    got = B.conv_wgrad_approx_topk(d, Xg, dYg, k, idx_out=idk).cpu().numpy()
    want, want_idx, _ = oracle.wgrad_approx_topk(g, X, dY, k)
    assert np.array_equal(idk.cpu().numpy(), want_idx)
    assert normwise_err(got, want) <= TOL[dtype]
    Xl = oracle.x_to_nhwc(X)
    Xlg = to_gpu(Xl)
    assert normwise_err(B.conv_wgrad_approx_nhwc(d, Xlg, dYg, layout).cpu().numpy(),
                        oracle.wgrad_approx_nhwc(g, Xl, dY, 1.0, layout)[0]) <= TOL[dtype]
    assert normwise_err(B.conv_wgrad_exact_nhwc(d, Xlg, dYg, layout).cpu().numpy(),
                        oracle.wgrad_exact_nhwc(g, Xl, dY, layout)) <= TOL[dtype]


@pytest.mark.parametrize("seed", range(8))
def test_random_stack_and_mask_through_schedule_run(seed):
    """A random stack (up to 44 layers drawn from a few shapes, so that groups of more than eight layers, more than six
    groups and more than 32 reductions occur) under a random method mask, every layer against the oracle."""
    import torch
    from paper_1908_05460_amd import schedule as sch
    rng = np.random.default_rng(4000 + seed)
    dtype = "bf16" if seed % 3 == 2 else "fp32"
    N = int(rng.integers(2, 24))
    pool = []
    while len(pool) < int(rng.integers(1, 9)) or not pool:
        hw = int(rng.choice([2, 4, 8, 16, 32, 7]))
        C = int(rng.choice([3, 16, 32, 64])); K = int(rng.choice([16, 32, 64, 128]))
        st = int(rng.choice([1, 1, 2])) if hw >= 8 else 1
        if N * K * hw * hw * C * 9 <= 6e7:
            pool.append((C, hw, K, st))
    nl = int(rng.integers(1, 45))
    layers = [pool[int(rng.integers(0, len(pool)))] for _ in range(nl)]
    methods = rng.integers(0, 4, nl).astype(np.uint8)
    descs = [B.desc(N, C, hw, hw, K, stride=st, dtype=B.BF16 if dtype == "bf16" else B.F32) for (C, hw, K, st) in layers]
    data = [rand_inputs(d, 100 * seed + i, dtype) for i, d in enumerate(descs)]
    dWs = [torch.full((d.K, d.C, 3, 3), float("nan"), device="cuda") for d in descs]
    s = B.Schedule(descs, [to_gpu(x) for x, _ in data], [to_gpu(y) for _, y in data], dWs)
    ws = B.alloc_workspace(s.workspace_bytes(methods))
    rseed, offset, sigma, scale = 77 + seed, int(rng.integers(0, 1 << 20)), 1 / 128, 0.25
    s.run(methods, ws, scale=scale, sigma=sigma, seed=rseed, offset=offset)
    off = offset
    for i, d in enumerate(descs):
        got = dWs[i].cpu().numpy()
        g = oracle_shape(d)
        if methods[i] == sch.EXACT:
            assert normwise_err(got, oracle.wgrad_exact(g, *data[i])) <= TOL[dtype], (i, layers[i])
        elif methods[i] == sch.APPROX:
            assert normwise_err(got, oracle.wgrad_approx(g, *data[i], scale=scale)[0]) <= TOL[dtype], (i, layers[i])
        elif methods[i] == sch.ZERO:
            assert not got.any(), (i, layers[i])
        else:
            assert np.abs(got.ravel() - oracle.random_normal(rseed, off, got.size, sigma)).max() <= 2e-5 * sigma, (i, layers[i])
        off += got.size
