"""GPU parity at the full benchmark sizes, through the same entry points and launch
configuration bench.py times.  The exact gradient is checked on sampled entries the oracle
computes one by one (each is a full N*Ho*Wo reduction); the approximation, whose oracle is
cheap, is checked on every entry, with the selected positions bit-exact."""
import numpy as np
import pytest

import oracle
from paper_1908_05460_amd import binding as B, inputs
from tests.gpu_util import TOL, check_select, normwise_err, oracle_shape, to_gpu

pytestmark = pytest.mark.gpu


def distinct_layers(workload):
    cfg, stack_fn, N, dtype = inputs.WORKLOADS[workload]
    seen, out = set(), []
    for i, l in enumerate(stack_fn()):
        key = (l.C, l.K, l.H, l.stride)
        if key not in seen:
            seen.add(key)
            out.append(pytest.param(workload, i, id=f"{workload}-{l.name}"))
    return out


CASES = (distinct_layers("single3x3_n16_fp32") + distinct_layers("resnet20_n128_fp32")
         + distinct_layers("vgg19_n128_fp32") + distinct_layers("vgg19_n512_bf16"))


@pytest.mark.parametrize("workload,index", CASES)
def test_layer_at_benchmark_size(workload, index):
    import torch
    cfg, stack_fn, N, dtype = inputs.WORKLOADS[workload]
    layer = stack_fn()[index]
    X, dY = inputs.make_layer_inputs(layer, N, config=cfg, batch=0, layer_index=index, dtype=dtype)
    d = B.desc_for(layer, N, dtype)
    g = oracle_shape(d)
    Xg, dYg = to_gpu(X), to_gpu(dY)
    ws = B.alloc_workspace(max(B.workspace_bytes(d, B.EXACT), B.workspace_bytes(d, B.APPROX)))

    # exact: sampled entries (corners included), error relative to the largest sampled |dW|
    got = B.conv_wgrad_exact(d, Xg, dYg, ws=ws).cpu().numpy().ravel()
    total = got.size
    rng = np.random.default_rng(index)
    pick = np.unique(np.concatenate([[0, total - 1, total // 2], rng.integers(0, total, 509)]))
    want = oracle.wgrad_exact_at(g, X, dY, pick)
    scale = np.abs(want).max()
    assert np.abs(got[pick].astype(np.float64) - want).max() <= TOL[dtype] * scale
    assert np.isfinite(got).all()

    # approximation: everything
    idx = torch.empty((N, layer.K), dtype=torch.int32, device="cuda")
    S = torch.empty((N, layer.K), dtype=torch.float32, device="cuda")
    got_a = B.conv_wgrad_approx(d, Xg, dYg, scale=1 / 128, idx_out=idx, sum_out=S, ws=ws).cpu().numpy()
    want_a, _, _ = oracle.wgrad_approx(g, X, dY, scale=1 / 128)
    check_select(d, dY, idx.cpu().numpy(), S.cpu().numpy())
    assert normwise_err(got_a, want_a) <= TOL[dtype]


@pytest.mark.parametrize("workload", ["resnet20_n128_fp32", "vgg19_n128_fp32", "vgg19_n512_bf16"])
def test_whole_stack_through_schedule_run_matches_per_layer_oracle_samples(workload):
    """The launch path bench.py uses: one conv_wgrad_schedule_run per method over the stack; then a mask that
    mixes the methods (every other layer approximated), as the schedule sweep runs it."""
    import torch
    from paper_1908_05460_amd import schedule as sch
    cfg, stack_fn, N, dtype = inputs.WORKLOADS[workload]
    stack = stack_fn()
    descs = [B.desc_for(l, N, dtype) for l in stack]
    data = [inputs.make_layer_inputs(l, N, cfg, 0, i, dtype) for i, l in enumerate(stack)]
    Xs = [to_gpu(x) for x, _ in data]; dYs = [to_gpu(y) for _, y in data]
    dWs = [torch.empty((l.K, l.C, 3, 3), device="cuda") for l in stack]
    s = B.Schedule(descs, Xs, dYs, dWs)
    exact = np.full(len(stack), sch.EXACT, np.uint8)
    approx = np.full(len(stack), sch.APPROX, np.uint8)
    mixed = exact.copy(); mixed[1::2] = sch.APPROX
    ws = B.alloc_workspace(max(s.workspace_bytes(m) for m in (exact, approx, mixed)))
    s.run(exact, ws)
    ex = [t.cpu().numpy().ravel().copy() for t in dWs]
    s.run(approx, ws, scale=1.0)
    ap = [t.cpu().numpy().copy() for t in dWs]
    s.run(mixed, ws, scale=1.0)
    mx = [t.cpu().numpy().copy() for t in dWs]
    rng = np.random.default_rng(5)
    for i, l in enumerate(stack):
        g = oracle_shape(descs[i])
        pick = rng.integers(0, ex[i].size, 24)
        want = oracle.wgrad_exact_at(g, data[i][0], data[i][1], pick)
        bound = TOL[dtype] * max(np.abs(want).max(), np.abs(ex[i]).max())
        assert np.abs(ex[i][pick] - want).max() <= bound, l.name
        want_a = oracle.wgrad_approx(g, data[i][0], data[i][1])[0]
        assert normwise_err(ap[i], want_a) <= TOL[dtype], l.name
        if mixed[i] == sch.APPROX:
            assert normwise_err(mx[i], want_a) <= TOL[dtype], l.name
        else:
            assert np.abs(mx[i].ravel()[pick] - want).max() <= bound, l.name
