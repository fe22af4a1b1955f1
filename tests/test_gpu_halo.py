"""K / V given as owned rows plus a separate halo tensor (Section 3.1, Algorithm 1): the results
must be bitwise those of the run on the concatenated tensors, and match the fp64 oracle."""
import numpy as np
import pytest
import torch

import gen
from helpers import TOL, Problem, assert_close, run_gpu, to_f64, to_torch

pytestmark = pytest.mark.gpu


def run_split(p: Problem, n_local, plan_kwargs=None, lean=False):
    import paper_2604_16715_amd as gta
    indptr = torch.from_numpy(p.indptr).cuda()
    indices = torch.from_numpy(p.indices).cuda()
    kw = dict(keep_dz_min_nnz=1)
    kw.update(plan_kwargs or {})
    plan = gta.gta_plan_create(indptr, indices, p.n_src, validate=True, **kw)
    Q, K, V, dO = (to_torch(getattr(p, k)) for k in ("Q", "K", "V", "dO"))
    # separate allocations (clones), not views of one tensor
    Kl, Vl = K[:n_local].clone(), V[:n_local].clone()
    Kh = K[n_local:].clone() if n_local < p.n_src else None
    Vh = V[n_local:].clone() if n_local < p.n_src else None
    out, lse = gta.gta_attn_fwd_halo(plan, Q, Kl, Vl, Kh, Vh)
    dQ, dKl, dVl, dKh, dVh = gta.gta_attn_bwd_halo(plan, Q, Kl, Vl, Kh, Vh, out, lse, dO, lean_scratch=lean)
    torch.cuda.synchronize()
    cat = lambda a, b: a if b is None else torch.cat([a, b], dim=0)
    return out, lse, dQ, cat(dKl, dKh), cat(dVl, dVh)


@pytest.mark.parametrize("name,shrink,kw", [
    ("partition", 16, None),                                  # owned + halo sources, bf16 [.,4,64]
    ("partition", 64, dict(wave_max_deg=16, hub_chunk=64)),   # hub rows split into chunks on both sides
    ("tiny", 1, None),                                        # fp32
])
@pytest.mark.parametrize("lean", [False, True])
def test_halo_pointers_match_concatenated_run(name, shrink, kw, lean):
    w = gen.workload(name, shrink)
    p = Problem.from_workload(w)
    n_local = p.n_dst if p.n_src > p.n_dst else (2 * p.n_src) // 3
    print(f"halo case {name}/{shrink} n_src={p.n_src} n_local={n_local} lean={lean} plan={kw}", flush=True)
    ref = run_gpu(p, plan_kwargs=kw, lean_scratch=lean)
    out, lse, dQ, dK, dV = run_split(p, n_local, kw, lean)
    dQr, dKr, dVr = ref["raw"]
    assert torch.equal(out, ref["raw_out"]) and torch.equal(lse, ref["raw_lse"])
    assert torch.equal(dQ, dQr) and torch.equal(dK, dKr) and torch.equal(dV, dVr)
    tol = TOL[p.dtype]
    o_out, _ = p.oracle_forward()
    o_dQ, o_dK, o_dV = p.oracle_backward()
    assert_close("out", to_f64(out), o_out, tol)
    assert_close("dQ", to_f64(dQ), o_dQ, tol)
    assert_close("dK", to_f64(dK), o_dK, tol)
    assert_close("dV", to_f64(dV), o_dV, tol)


def test_halo_degenerate_splits_and_errors():
    import paper_2604_16715_amd as gta
    indptr, indices = gen.random_csr(300, 400, 4000, seed=77, allow_dup=True, sort_rows=False)
    p = Problem.random(indptr, indices, 400, 4, 16, "f32", seed=9)
    ref = run_gpu(p)
    for n_local in (0, 1, 399, 400):   # everything halo, one owned row, one halo row, no halo
        print(f"halo split n_local={n_local}", flush=True)
        out, lse, dQ, dK, dV = run_split(p, n_local)
        dQr, dKr, dVr = ref["raw"]
        assert torch.equal(out, ref["raw_out"]) and torch.equal(dQ, dQr)
        assert torch.equal(dK, dKr) and torch.equal(dV, dVr)
    # missing halo tensor while n_local < n_src
    plan = ref["plan"]
    Q, K, V = (to_torch(getattr(p, k)) for k in ("Q", "K", "V"))
    with pytest.raises(gta.GtaError):
        gta.gta_attn_fwd_halo(plan, Q, K[:100].clone(), V[:100].clone(), None, None)
