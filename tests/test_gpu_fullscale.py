"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (default
plan): the oracle runs the whole workload and every element of out, lse, dQ, dK and dV is
compared (2.4 M - 8.4 M rows, 49 M - 140 M stored entries per workload); the dense kernels of the layer run at
the same row count and are compared on sampled rows."""
import pytest

import gen
from helpers import Problem, whole_parity

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["large", "partition", "skew"])
def test_full_size_whole_tensor_parity(name):
    print(f"whole-tensor case {name}: generating", flush=True)
    w = gen.workload(name)
    whole_parity(Problem.from_workload(w), name, w.nnz)


def test_full_size_dense_projections():
    """The layer's dense kernels at the benchmark's row count (n = 2.45 M, d = 256, bfloat16: 1.25 GB per
    tensor, offsets past 2^30 bytes): Q, K, V from one read of X (Eq. 3), X W_o + Y (Eq. 5), the four-term
    input gradient and the four weight gradients.  Row-wise results are compared on the first and last rows
    and on random rows, each against its own float64 product; two of the weight gradients whole."""
    import numpy as np
    import torch

    import paper_2604_16715_amd as gta
    from helpers import assert_close, to_f64, to_torch
    from oracle import dense_ref

    n, d = 2_450_000, 256
    print(f"dense full-size case n={n} d={d}: generating", flush=True)
    f = lambda a: gen.bf16_bits_to_f32(a).astype(np.float64)
    Xs = [gen.normal((n, d), "bf16", 5, 60 + i) for i in range(4)]
    Ws = []
    for i in range(4):   # weights of magnitude 1/16, truncated to bf16
        w32 = (gen.bf16_bits_to_f32(gen.normal((d, d), "bf16", 5, 70 + i)) * 0.0625).astype(np.float32)
        Ws.append((w32.view(np.uint32) >> 16).astype(np.uint16))
    Xd, Wd = [to_torch(a) for a in Xs], [to_torch(a) for a in Ws]
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([np.arange(256), np.arange(n - 256, n), rng.integers(0, n, 4096)]))
    rows_t = torch.from_numpy(rows).cuda()
    pick = lambda t: to_f64(t[rows_t])
    Xr, Wf = [f(a[rows]) for a in Xs], [f(a) for a in Ws]

    print("  Q, K, V in one launch", flush=True)
    Q, K, V = gta.gta_linear_group([Xd[0]], Wd[:3])
    for name, got, W in zip("QKV", (Q, K, V), Wf[:3]):
        assert_close(name, pick(got), dense_ref.linear(Xr[0], W), 2e-2)
    del Q, K, V
    print("  X W_o + Y", flush=True)
    out = gta.gta_linear(Xd[0], Wd[3], Xd[1])
    assert_close("X W_o + Y", pick(out), dense_ref.linear(Xr[0], Wf[3], Xr[1]), 2e-2)
    del out
    print("  dX as one four-term sum", flush=True)
    (dX,) = gta.gta_linear_group(Xd, Wd, trans_w=True)
    ref = sum(dense_ref.linear(x, w, trans_w=True) for x, w in zip(Xr, Wf))
    assert_close("dX", pick(dX), ref, 2e-2)
    del dX
    print("  four weight gradients in one launch", flush=True)
    dWs = gta.gta_linear_dw_group([Xd[0]] * 4, Xd)
    torch.cuda.synchronize()
    X0 = f(Xs[0])
    for k in (1, 3):
        print(f"  float64 X^T dY[{k}]", flush=True)
        assert_close(f"dW[{k}]", to_f64(dWs[k]), dense_ref.linear_dw(X0, f(Xs[k])), 1e-4)
    for k in range(4):   # bit-identical to the single-product entry point
        assert torch.equal(dWs[k], gta.gta_linear_dw(Xd[0], Xd[k]))
    torch.cuda.synchronize()


def test_full_size_layer():
    """One whole layer forward + backward (Eq. 3-5 and their gradients) on all of `large`, hidden 256, against
    the float64 layer reference: Q, Y, X', dX and the four weight gradients, every element."""
    import test_gpu_layer
    test_gpu_layer.test_layer_forward_backward("large", 1, 8, 32)
