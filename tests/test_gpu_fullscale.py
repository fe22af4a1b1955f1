"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (default
plan).  The oracle cannot run the whole problem in seconds, so it computes sampled output rows
one sub-problem at a time:

* a destination row's out / lse / dQ depend only on that row's entries, so the sub-problem is
  the sampled rows with all their entries (sources renumbered compactly);
* a source row's dK / dV need every entry that points to it and, for each of those, the whole
  softmax row of its destination; the sub-problem is every destination row that references a
  sampled source, with all its entries.

Two identities that hold at any size are checked on the complete GPU outputs as well.
"""
import numpy as np
import pytest
import torch

import gen
import oracle
from helpers import TOL, Problem, assert_close, assert_lse_close, run_gpu

pytestmark = pytest.mark.gpu


def subproblem(p: Problem, rows: np.ndarray):
    """Rows `rows` of the problem with all their entries; sources renumbered compactly."""
    rows = np.asarray(rows, dtype=np.int64)
    deg = (p.indptr[rows + 1] - p.indptr[rows]).astype(np.int64)
    indptr = np.zeros(len(rows) + 1, dtype=np.int64)
    indptr[1:] = np.cumsum(deg)
    take = np.concatenate([np.arange(p.indptr[r], p.indptr[r + 1]) for r in rows]) if len(rows) else np.zeros(0, np.int64)
    uniq, inv = np.unique(p.indices[take], return_inverse=True)
    f64 = lambda x: gen.as_f32(x).astype(np.float64)
    return dict(indptr=indptr, indices=inv.astype(np.int32), uniq=uniq, Q=f64(p.Q[rows]), dO=f64(p.dO[rows]),
                K=f64(p.K[uniq]), V=f64(p.V[uniq]))


def sample_rows(ptr: np.ndarray, count: int, rng) -> np.ndarray:
    """The three longest rows plus rows drawn from every power-of-two degree range."""
    deg = np.diff(ptr)
    picks = list(np.argsort(deg)[-3:])
    cls = np.ceil(np.log2(np.maximum(deg, 1))).astype(np.int64)
    cls[deg == 0] = -1
    for c in np.unique(cls):
        members = np.flatnonzero(cls == c)
        picks.extend(rng.choice(members, size=min(len(members), max(2, count // 20)), replace=False))
    return np.unique(np.array(picks, dtype=np.int64))


@pytest.mark.parametrize("name", ["large", "partition", "skew"])
def test_full_size_sampled_parity(name):
    print(f"full-size case {name}: generating", flush=True)
    w = gen.workload(name)
    p = Problem.from_workload(w)
    tol = TOL[p.dtype]
    print(f"full-size case {name}: n_dst={p.n_dst} n_src={p.n_src} nnz={w.nnz}; GPU fwd+bwd", flush=True)
    res = run_gpu(p)
    rng = np.random.Generator(np.random.Philox(w.seed))

    # ---- destination rows: out, lse, dQ
    rows = sample_rows(p.indptr, 120, rng)
    sp = subproblem(p, rows)
    print(f"full-size case {name}: oracle on {len(rows)} destination rows, {int(sp['indptr'][-1])} entries", flush=True)
    out, lse = oracle.forward(sp["indptr"], sp["indices"], sp["Q"], sp["K"], sp["V"])
    dQ, _, _ = oracle.backward(sp["indptr"], sp["indices"], sp["Q"], sp["K"], sp["V"], sp["dO"])
    assert_close("out", res["out"][rows], out, tol)
    assert_lse_close(res["lse"][rows], lse, tol)
    assert_close("dQ", res["dQ"][rows], dQ, tol)

    # ---- source rows: dK, dV
    t_deg_ptr = np.zeros(p.n_src + 1, dtype=np.int64)
    t_deg_ptr[1:] = np.cumsum(np.bincount(p.indices, minlength=p.n_src))
    srcs = sample_rows(t_deg_ptr, 60, rng)
    if p.n_src > p.n_dst:   # make sure halo rows are sampled
        srcs = np.unique(np.concatenate([srcs, rng.integers(p.n_dst, p.n_src, size=20)]))
    hit = np.flatnonzero(np.isin(p.indices, srcs))
    dst_rows = np.unique(np.searchsorted(p.indptr, hit, side="right") - 1)
    sp = subproblem(p, dst_rows)
    print(f"full-size case {name}: oracle on {len(srcs)} source rows via {len(dst_rows)} destination rows, "
          f"{int(sp['indptr'][-1])} entries", flush=True)
    _, dK, dV = oracle.backward(sp["indptr"], sp["indices"], sp["Q"], sp["K"], sp["V"], sp["dO"])
    pos = np.searchsorted(sp["uniq"], srcs)
    present = (pos < len(sp["uniq"])) & (sp["uniq"][np.minimum(pos, len(sp["uniq"]) - 1)] == srcs)
    ref_dK = np.zeros((len(srcs),) + dK.shape[1:])
    ref_dV = np.zeros_like(ref_dK)
    ref_dK[present], ref_dV[present] = dK[pos[present]], dV[pos[present]]
    assert_close("dK", res["dK"][srcs], ref_dK, tol)
    assert_close("dV", res["dV"][srcs], ref_dV, tol)

    # ---- identities on the complete outputs (fp64 reductions of the GPU tensors)
    dQ_t, dK_t, dV_t = res["raw"]
    Q_t = torch.from_numpy(gen.as_f32(p.Q)).cuda().double()
    K_t = torch.from_numpy(gen.as_f32(p.K)).cuda().double()
    dO_t = torch.from_numpy(gen.as_f32(p.dO)).cuda().double()
    nonempty = torch.from_numpy(np.diff(p.indptr) > 0).cuda()
    lhs = dV_t.double().sum(dim=0)
    rhs = (dO_t * nonempty[:, None, None]).sum(dim=0)
    scale_ref = dO_t.abs().sum(dim=0)          # rounding of ~n terms grows like the absolute sum
    assert torch.all((lhs - rhs).abs() <= tol * scale_ref), "sum_j dV_j != sum_i dY_i"
    qdq = (Q_t * dQ_t.double()).sum(dim=(0, 2))
    kdk = (K_t * dK_t.double()).sum(dim=(0, 2))
    mag = (Q_t * dQ_t.double()).abs().sum(dim=(0, 2))
    assert torch.all((qdq - kdk).abs() <= tol * mag), "sum q.dQ != sum k.dK"
