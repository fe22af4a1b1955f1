"""One full Sparse Graph Attention layer (projections on the matrix cores + fused attention) against
the float64 layer reference, forward and backward."""
import numpy as np
import pytest
import torch

import gen
from helpers import assert_close, to_f64, to_torch
from oracle import layer_ref

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,shrink,heads,head_dim", [("tiny", 1, 4, 16), ("mid", 16, 8, 16), ("large", 128, 8, 32)])
def test_layer_forward_backward(name, shrink, heads, head_dim):
    import paper_2604_16715_amd as gta
    w = gen.workload(name, shrink)
    n, d = w.n_dst, heads * head_dim
    print(f"layer case {name}/{shrink} n={n} nnz={w.nnz} d={d}", flush=True)
    bits = lambda shape, stream, scale: ((gen.bf16_bits_to_f32(gen.normal(shape, "bf16", w.seed, stream)) * scale)
                                         .astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    X, dXout = bits((n, d), 2, 1.0), bits((n, d), 5, 1.0)
    Ws = [bits((d, d), 10 + k, 0.125) for k in range(4)]    # ~N(0, 1/64): scores of order one
    f64 = lambda a: gen.bf16_bits_to_f32(a).astype(np.float64)
    plan = gta.gta_plan_create(torch.from_numpy(w.indptr).cuda(), torch.from_numpy(w.indices).cuda(), n, keep_dz_min_nnz=1)
    Xd, dXd = to_torch(X), to_torch(dXout)
    Wd = [to_torch(a) for a in Ws]
    Xout, saved = gta.gta_sga_layer_fwd(plan, Xd, *Wd, heads)
    dX, dWq, dWk, dWv, dWo = gta.gta_sga_layer_bwd(plan, Xd, *Wd, saved, dXd, heads)
    torch.cuda.synchronize()
    ref_out, ref_saved = layer_ref.layer_forward(w.indptr, w.indices, f64(X), *[f64(a) for a in Ws], heads)
    ref = layer_ref.layer_backward(w.indptr, w.indices, f64(X), *[f64(a) for a in Ws], heads, f64(dXout))
    tol = 2e-2
    assert_close("Q", to_f64(saved["Q"]).reshape(n, heads, head_dim), ref_saved["Q"], tol)
    assert_close("Y", to_f64(saved["Y"]).reshape(n, heads, head_dim), ref_saved["Y"], tol)
    assert_close("X'", to_f64(Xout), ref_out, tol)
    for label, got, want in zip(("dX", "dWq", "dWk", "dWv", "dWo"), (dX, dWq, dWk, dWv, dWo), ref):
        assert_close(label, to_f64(got), want, tol)


@pytest.mark.parametrize("name,shrink,heads,head_dim", [("tiny", 1, 4, 16), ("mid", 4, 8, 16)])
def test_layer_forward_backward_f32(name, shrink, heads, head_dim):
    """The fp32 layer (the tiny and mid workloads are fp32), every tensor at the fp32 bar of 1e-5
    (measured: 4e-7 .. 1e-6 through projection, attention and projection)."""
    import paper_2604_16715_amd as gta
    w = gen.workload(name, shrink)
    n, d = w.n_dst, heads * head_dim
    print(f"layer f32 case {name}/{shrink} n={n} nnz={w.nnz} d={d}", flush=True)
    mk = lambda shape, stream, scale: (gen.normal(shape, "f32", w.seed, stream) * np.float32(scale)).astype(np.float32)
    X, dXout = mk((n, d), 2, 1.0), mk((n, d), 5, 1.0)
    Ws = [mk((d, d), 10 + k, 0.125) for k in range(4)]
    f64 = lambda a: a.astype(np.float64)
    plan = gta.gta_plan_create(torch.from_numpy(w.indptr).cuda(), torch.from_numpy(w.indices).cuda(), n, keep_dz_min_nnz=1)
    Xd, dXd = to_torch(X), to_torch(dXout)
    Wd = [to_torch(a) for a in Ws]
    Xout, saved = gta.gta_sga_layer_fwd(plan, Xd, *Wd, heads)
    dX, dWq, dWk, dWv, dWo = gta.gta_sga_layer_bwd(plan, Xd, *Wd, saved, dXd, heads)
    torch.cuda.synchronize()
    ref_out, ref_saved = layer_ref.layer_forward(w.indptr, w.indices, f64(X), *[f64(a) for a in Ws], heads)
    ref = layer_ref.layer_backward(w.indptr, w.indices, f64(X), *[f64(a) for a in Ws], heads, f64(dXout))
    tol = 1e-5
    assert_close("Q", to_f64(saved["Q"]).reshape(n, heads, head_dim), ref_saved["Q"], 1e-5)
    assert_close("Y", to_f64(saved["Y"]).reshape(n, heads, head_dim), ref_saved["Y"], tol)
    assert_close("X'", to_f64(Xout), ref_out, tol)
    for label, got, want in zip(("dX", "dWq", "dWk", "dWv", "dWo"), (dX, dWq, dWk, dWv, dWo), ref):
        assert_close(label, to_f64(got), want, tol)
