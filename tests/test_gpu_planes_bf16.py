"""bf16 inputs on 2x2 and 4x4 planes: the position-major matrix-core kernel, exact and through the sparsified
gradient of the approximation, single layers and layers of one shape folded into one launch, against the oracle
on every dW entry."""
import numpy as np
import pytest

import oracle
from paper_1908_05460_amd import binding as B
from tests.gpu_util import TOL, check_select, normwise_err, oracle_shape, rand_inputs, to_gpu

pytestmark = pytest.mark.gpu

# (N, C, HW, K): batches of 32 images and more, channel counts the tiles divide
SINGLE = [(32, 64, 2, 32), (64, 128, 2, 64), (96, 64, 2, 96), (32, 32, 4, 32), (64, 96, 4, 64), (160, 64, 4, 32)]


def desc(N, C, HW, K):
    return B.desc(N, C, HW, HW, K, R=3, S=3, pad=1, dtype=B.BF16)


@pytest.mark.parametrize("t", SINGLE)
def test_single_layer_exact_and_approx(t):
    import torch
    d = desc(*t)
    X, dY = rand_inputs(d, 31 + t[0] + t[2], "bf16")
    g = oracle_shape(d)
    got = B.conv_wgrad_exact(d, to_gpu(X), to_gpu(dY)).cpu().numpy()
    assert normwise_err(got, oracle.wgrad_exact(g, X, dY)) <= TOL["bf16"]
    idx = torch.empty((d.N, d.K), dtype=torch.int32, device="cuda")
    S = torch.empty((d.N, d.K), dtype=torch.float32, device="cuda")
    got = B.conv_wgrad_approx(d, to_gpu(X), to_gpu(dY), scale=0.5, idx_out=idx, sum_out=S).cpu().numpy()
    check_select(d, dY, idx.cpu().numpy(), S.cpu().numpy())
    assert normwise_err(got, oracle.wgrad_approx(g, X, dY, scale=0.5)[0]) <= TOL["bf16"]


@pytest.mark.parametrize("hw,layers", [(2, 3), (4, 3)])
def test_layers_of_one_shape_in_one_launch(hw, layers):
    """Three layers of 512 -> 512 channels folded into one launch by a schedule run."""
    import torch
    d = desc(32, 512, hw, 512)
    g = oracle_shape(d)
    data = [rand_inputs(d, 900 + 10 * hw + i, "bf16") for i in range(layers)]
    dWs = [torch.full((512, 512, 3, 3), float("nan"), device="cuda") for _ in range(layers)]
    S = B.Schedule([d] * layers, [to_gpu(x) for x, _ in data], [to_gpu(y) for _, y in data], dWs)
    for method, ref in ((B.EXACT, lambda x, y: oracle.wgrad_exact(g, x, y)),
                        (B.APPROX, lambda x, y: oracle.wgrad_approx(g, x, y)[0])):
        mask = np.full(layers, method, np.uint8)
        ws = B.alloc_workspace(S.workspace_bytes(mask))
        for w in dWs:
            w.fill_(float("nan"))
        S.run(mask, ws)
        torch.cuda.synchronize()
        for (x, y), w in zip(data, dWs):
            assert normwise_err(w.cpu().numpy(), ref(x, y)) <= TOL["bf16"]
