"""GPU parity at the full benchmark sizes, through the same entry points and launch
configuration bench.py times.  Every entry of every dW tensor is compared with the oracle,
for the exact gradient (Section 2.4's definition) and for the approximation (Algorithm 1),
whose selected positions must be bit-exact."""
import numpy as np
import pytest

import oracle
from paper_1908_05460_amd import binding as B, inputs
from tests.gpu_util import TOL, check_select, elementwise_pass_rate, normwise_err, oracle_shape, to_gpu

pytestmark = pytest.mark.gpu

_ORACLE_EXACT = {}      # (workload, layer index) -> the oracle's full exact dW; both tests below use batch 0


def oracle_exact_full(workload, index, g, X, dY):
    key = (workload, index)
    if key not in _ORACLE_EXACT:
        _ORACLE_EXACT[key] = oracle.wgrad_exact(g, X, dY)
    return _ORACLE_EXACT[key]


def assert_exact_everywhere(got, want, dtype, what):
    """max |gpu - oracle| over ALL entries against tol * max |oracle|; the element-wise pass rate
    of |g - o| <= tol*|o| + tol*rms(o) is printed as information (entries are cancelling sums)."""
    got = np.asarray(got, np.float64).reshape(want.shape)
    assert np.isfinite(got).all(), what
    err = normwise_err(got, want)
    print(f"{what}: normwise {err:.2e}, element-wise pass rate {elementwise_pass_rate(got, want, TOL[dtype]):.6f}"
          f" over {want.size} entries")
    assert err <= TOL[dtype], (what, err)


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

    # exact: every entry
    got = B.conv_wgrad_exact(d, Xg, dYg, ws=ws).cpu().numpy()
    assert_exact_everywhere(got, oracle_exact_full(workload, index, g, X, dY), dtype, f"{workload} {layer.name} single call")

    # approximation: everything
    idx = torch.empty((N, layer.K), dtype=torch.int32, device="cuda")
    S = torch.empty((N, layer.K), dtype=torch.float32, device="cuda")
    got_a = B.conv_wgrad_approx(d, Xg, dYg, scale=1 / 128, idx_out=idx, sum_out=S, ws=ws).cpu().numpy()
    want_a, _, _ = oracle.wgrad_approx(g, X, dY, scale=1 / 128)
    check_select(d, dY, idx.cpu().numpy(), S.cpu().numpy())
    assert normwise_err(got_a, want_a) <= TOL[dtype]


@pytest.mark.parametrize("workload", ["resnet20_n128_fp32", "vgg19_n128_fp32", "vgg19_n512_bf16"])
def test_whole_stack_through_schedule_run_matches_the_oracle_everywhere(workload):
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
    ex = [t.cpu().numpy().copy() for t in dWs]
    s.run(approx, ws, scale=1.0)
    ap = [t.cpu().numpy().copy() for t in dWs]
    s.run(mixed, ws, scale=1.0)
    mx = [t.cpu().numpy().copy() for t in dWs]
    for i, l in enumerate(stack):
        g = oracle_shape(descs[i])
        want = oracle_exact_full(workload, i, g, data[i][0], data[i][1])
        assert_exact_everywhere(ex[i], want, dtype, f"{workload} {l.name} all-exact run")
        want_a = oracle.wgrad_approx(g, data[i][0], data[i][1])[0]
        assert normwise_err(ap[i], want_a) <= TOL[dtype], l.name
        if mixed[i] == sch.APPROX:
            assert normwise_err(mx[i], want_a) <= TOL[dtype], l.name
        else:
            assert_exact_everywhere(mx[i], want, dtype, f"{workload} {l.name} mixed run")
