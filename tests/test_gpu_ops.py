"""The standalone operators (SDDMM, edge softmax and its backward, SpMM, transposed SpMM) against
the oracle's, and the unfused composition against the fused path's oracle."""
import numpy as np
import pytest
import torch

import gen
import oracle
from helpers import TOL, Problem, assert_close, assert_lse_close, to_f64, to_torch

pytestmark = pytest.mark.gpu


def run_ops(p: Problem, plan_kwargs, tag):
    import paper_2604_16715_amd as gta
    print(f"ops case {tag}: n_dst={p.n_dst} n_src={p.n_src} nnz={int(p.indptr[-1])} shape={p.Q.shape[1:]} "
          f"dtype={p.dtype} plan={plan_kwargs}", flush=True)
    tol = TOL[p.dtype]
    plan = gta.gta_plan_create(torch.from_numpy(p.indptr).cuda(), torch.from_numpy(p.indices).cuda(), p.n_src,
                               **(plan_kwargs or {}))
    Q, K, V, dO = (to_torch(getattr(p, k)) for k in ("Q", "K", "V", "dO"))
    Qh, Kh, Vh, dOh = (p.f64(k) for k in ("Q", "K", "V", "dO"))
    D = Q.shape[2]
    scale = 1.0 / np.sqrt(D)
    E = int(p.indptr[-1])
    # forward: SDDMM -> softmax -> SpMM
    Z = gta.gta_sddmm(plan, Q, K)
    Zr = oracle.sddmm(p.indptr, p.indices, Qh, Kh)
    assert_close("Z", to_f64(Z), Zr, 1e-5)   # inputs exact in either dtype, fp32 accumulate
    U, lse = gta.gta_edge_softmax(plan, Z, scale)
    Ur, lser = oracle.edge_softmax(p.indptr, Zr, scale)
    assert_close("U", to_f64(U), Ur, 1e-5)
    assert_lse_close(to_f64(lse), lser, 1e-5)
    Y = gta.gta_spmm(plan, U, V)
    Yr = oracle.spmm(p.indptr, p.indices, Ur, Vh)
    assert_close("Y", to_f64(Y), Yr, tol)
    # the composition equals the attention forward
    out_ref, _ = p.oracle_forward()
    assert_close("Y vs fused definition", to_f64(Y), out_ref, tol)
    # backward operators
    dV = gta.gta_spmm(plan, U, dO, transposed=True)
    assert_close("dV", to_f64(dV), oracle.spmm(p.indptr, p.indices, Ur, dOh, p.n_src, transposed=True), tol)
    dU = gta.gta_sddmm(plan, dO, V)
    dUr = oracle.sddmm(p.indptr, p.indices, dOh, Vh)
    assert_close("dU", to_f64(dU), dUr, 1e-5)
    # the operator by itself: the oracle's operator on the very U and dU the GPU operator was given
    dZ = gta.gta_edge_softmax_bwd(plan, U, dU, scale)
    assert_close("dZ", to_f64(dZ), oracle.edge_softmax_bwd(p.indptr, to_f64(U), to_f64(dU), scale), 1e-5)
    dQ = gta.gta_spmm(plan, dZ, K)
    dK = gta.gta_spmm(plan, dZ, Q, transposed=True)
    dQr, dKr, dVr = p.oracle_backward()
    assert_close("dQ", to_f64(dQ), dQr, tol)
    assert_close("dK", to_f64(dK), dKr, tol)
    assert_close("dV vs definition", to_f64(dV), dVr, tol)
    torch.cuda.synchronize()
    assert E == Z.shape[0]


@pytest.mark.parametrize("name,shrink,kw", [
    ("tiny", 1, None), ("tiny", 1, dict(wave_max_deg=8, hub_chunk=32)), ("mid", 2, None),
    ("large", 32, dict(wave_max_deg=32, hub_chunk=128)), ("partition", 32, None), ("skew", 64, None),
])
def test_operators_on_workloads(name, shrink, kw):
    run_ops(Problem.from_workload(gen.workload(name, shrink)), kw, f"{name}/{shrink}")


def test_operators_edge_cases():
    import paper_2604_16715_amd as gta
    # unsorted rows with duplicates, empty rows, halo sources
    indptr, indices = gen.random_csr(300, 500, 4000, seed=12, allow_dup=True, sort_rows=False)
    run_ops(Problem.random(indptr, indices, 500, 2, 64, "bf16", 3), dict(wave_max_deg=16, hub_chunk=16), "ragged")
    # sliced rows: 2048-byte rows (two slices) and 3 heads (three slices)
    run_ops(Problem.random(indptr, indices, 500, 8, 64, "f32", 4), dict(wave_max_deg=16, hub_chunk=16), "wide rows")
    # no entries
    p = Problem.random(np.zeros(5, dtype=np.int64), np.zeros(0, dtype=np.int32), 6, 4, 16, "f32", 1)
    run_ops(p, None, "empty")
    # argument errors
    plan = gta.gta_plan_create(torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda(), 500)
    Z = torch.zeros((int(indptr[-1]), 3), device="cuda")
    with pytest.raises(gta.GtaError):
        gta.gta_edge_softmax(plan, Z, 1.0)          # heads not a power of two
    Z = torch.zeros((int(indptr[-1]), 4), device="cuda")
    with pytest.raises(gta.GtaError):
        gta.gta_edge_softmax(plan, Z, 0.0)          # scale must be given


@pytest.mark.parametrize("heads", [1, 2, 4, 8, 16, 32, 64])
@pytest.mark.parametrize("kw", [None, dict(wave_max_deg=8, hub_chunk=32)])
def test_edge_softmax_all_head_counts(heads, kw):
    """Both access widths (4 bytes per lane for H < 4, 16 bytes for H >= 4, also on an unaligned
    view) and all three team sizes, against the oracle's operators."""
    import oracle
    import paper_2604_16715_amd as gta
    print(f"edge softmax heads={heads} plan={kw}", flush=True)
    indptr, indices = gen.random_csr(400, 500, 9000, seed=40 + heads, allow_dup=True, sort_rows=False)
    indptr = indptr.copy()
    E = int(indptr[-1])
    rng = np.random.Generator(np.random.Philox(heads))
    Z = (3.0 * rng.standard_normal((E, heads))).astype(np.float32)
    dU = rng.standard_normal((E, heads)).astype(np.float32)
    scale = 0.7
    plan = gta.gta_plan_create(torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda(), 500, **(kw or {}))
    ref_U, ref_lse = oracle.edge_softmax(indptr, Z.astype(np.float64), scale)
    ref_dZ = oracle.edge_softmax_bwd(indptr, ref_U, dU.astype(np.float64), scale)
    Zd, dUd = torch.from_numpy(Z).cuda(), torch.from_numpy(dU).cuda()
    U, lse = gta.gta_edge_softmax(plan, Zd, scale)
    dZ = gta.gta_edge_softmax_bwd(plan, torch.from_numpy(ref_U.astype(np.float32)).cuda(), dUd, scale)
    torch.cuda.synchronize()
    assert_close("U", to_f64(U), ref_U, 1e-5)
    assert_lse_close(to_f64(lse), ref_lse, 1e-5)
    assert_close("dZ", to_f64(dZ), ref_dZ, 1e-5)
    # the same through buffers that are only 4-byte aligned
    pad = torch.empty(E * heads + 1, dtype=torch.float32, device="cuda")
    Zu = pad[1:].view(E, heads)
    Zu.copy_(Zd)
    U2, lse2 = gta.gta_edge_softmax(plan, Zu, scale)
    torch.cuda.synchronize()
    assert_close("U (4-byte path)", to_f64(U2), ref_U, 1e-5)     # another summation order than the 16-byte path
    assert_lse_close(to_f64(lse2), ref_lse, 1e-5)
