"""Shared helpers for the GPU parity tests: upload seeded inputs, run the library through its
C ABI binding, run the oracle on the same inputs, and measure errors."""
from __future__ import annotations

import numpy as np
import torch

import gen
import oracle

TOL = {"f32": 1e-5, "bf16": 2e-2}   # normwise relative tolerances


def to_torch(x: np.ndarray, device="cuda") -> torch.Tensor:
    """Storage array (float32, or uint16 holding bfloat16 bits) -> device tensor."""
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(x).to(device)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def rel_errors(got: np.ndarray, ref: np.ndarray):
    """(max-norm error / max|ref|, 2-norm error / 2-norm ref)."""
    diff = got - ref
    den_max = max(float(np.max(np.abs(ref))) if ref.size else 0.0, 1e-300)
    den_l2 = max(float(np.sqrt(np.sum(ref * ref))) if ref.size else 0.0, 1e-300)
    if ref.size == 0:
        return 0.0, 0.0
    return float(np.max(np.abs(diff))) / den_max, float(np.sqrt(np.sum(diff * diff))) / den_l2


def assert_close(name, got, ref, tol):
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{name}: non-finite values"
    emax, el2 = rel_errors(got, ref)
    print(f"    {name}: max-norm rel {emax:.2e}, l2 rel {el2:.2e} (gate {tol:.0e})", flush=True)
    assert emax <= tol and el2 <= tol, f"{name}: max-norm rel {emax:.3e}, l2 rel {el2:.3e} > {tol:.1e}"
    return emax, el2


def assert_lse_close(got, ref, tol):
    empty = np.isinf(ref)
    assert np.array_equal(np.isneginf(got), empty), "lse: -inf pattern differs"
    g, r = got[~empty], ref[~empty]
    assert np.all(np.abs(g - r) <= tol * np.maximum(1.0, np.abs(r))), \
        f"lse: max abs err {np.max(np.abs(g - r)) if g.size else 0:.3e}"


class Problem:
    """Inputs of one workload in storage precision (host) plus their exact float64 widening."""

    def __init__(self, indptr, indices, n_src, Q, K, V, dO, dtype):
        self.indptr = np.ascontiguousarray(indptr, dtype=np.int64)
        self.indices = np.ascontiguousarray(indices, dtype=np.int32)
        self.n_dst, self.n_src = len(indptr) - 1, n_src
        self.Q, self.K, self.V, self.dO = Q, K, V, dO
        self.dtype = dtype

    @classmethod
    def from_workload(cls, w: "gen.Workload"):
        return cls(w.indptr, w.indices, w.n_src, w.tensor("Q"), w.tensor("K"), w.tensor("V"),
                   w.tensor("dO"), w.dtype)

    @classmethod
    def random(cls, indptr, indices, n_src, heads, head_dim, dtype, seed):
        n_dst = len(indptr) - 1
        mk = lambda rows, stream: gen.normal((rows, heads, head_dim), dtype, seed, stream)
        return cls(indptr, indices, n_src, mk(n_dst, 2), mk(n_src, 3), mk(n_src, 4), mk(n_dst, 5), dtype)

    def f64(self, name):
        return gen.as_f32(getattr(self, name)).astype(np.float64)

    def oracle_forward(self, scale=None):
        return oracle.forward(self.indptr, self.indices, self.f64("Q"), self.f64("K"), self.f64("V"), scale)

    def oracle_backward(self, scale=None):
        return oracle.backward(self.indptr, self.indices, self.f64("Q"), self.f64("K"), self.f64("V"),
                               self.f64("dO"), scale)


def run_gpu(p: Problem, scale=0.0, plan_kwargs=None, backward=True, lean_scratch=False):
    """Plan + forward (+ backward) through the C ABI.  Returns dict of float64 host arrays + plan.
    lean_scratch selects the backward form that keeps nothing per stored entry."""
    import paper_2604_16715_amd as gta
    indptr = torch.from_numpy(p.indptr).cuda()
    indices = torch.from_numpy(p.indices).cuda()
    kw = dict(keep_dz_min_nnz=1)   # small test graphs must still run the dZ-keeping backward
    kw.update(plan_kwargs or {})
    plan = gta.gta_plan_create(indptr, indices, p.n_src, validate=True, **kw)
    Q, K, V, dO = (to_torch(getattr(p, k)) for k in ("Q", "K", "V", "dO"))
    out, lse = gta.gta_attn_fwd(plan, Q, K, V, scale)
    res = dict(plan=plan, out=to_f64(out), lse=to_f64(lse), raw_out=out, raw_lse=lse)
    if backward:
        dQ, dK, dV = gta.gta_attn_bwd(plan, Q, K, V, out, lse, dO, scale, lean_scratch=lean_scratch)
        res.update(dQ=to_f64(dQ), dK=to_f64(dK), dV=to_f64(dV), raw=(dQ, dK, dV))
    torch.cuda.synchronize()
    return res


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


def sampled_parity(p: Problem, name: str, seed: int, nnz: int, dst_count: int = 120, src_count: int = 60):
    """GPU forward + backward on the whole problem (default plan), oracle on sampled rows."""
    tol = TOL[p.dtype]
    print(f"full-size case {name}: n_dst={p.n_dst} n_src={p.n_src} nnz={nnz}; GPU fwd+bwd", flush=True)
    res = run_gpu(p)
    rng = np.random.Generator(np.random.Philox(seed))

    # ---- destination rows: out, lse, dQ
    rows = sample_rows(p.indptr, dst_count, rng)
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
    srcs = sample_rows(t_deg_ptr, src_count, rng)
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


def whole_parity(p: Problem, name: str, nnz: int):
    """GPU forward + backward on the whole problem in the benchmark's launch configuration (default
    plan), the oracle on the whole problem too; all five outputs compared element by element."""
    import time
    tol = TOL[p.dtype]
    print(f"whole-tensor case {name}: n_dst={p.n_dst} n_src={p.n_src} nnz={nnz}; GPU fwd+bwd", flush=True)
    res = run_gpu(p, plan_kwargs=dict(keep_dz_min_nnz=0))
    info = res["plan"].info()
    print(f"whole-tensor case {name}: plan has {int(info.n_chunked[0])}/{int(info.n_chunked[1])} chunked rows, "
          f"{int(info.n_hub[0])}/{int(info.n_hub[1])} split rows (dst/src side); widening inputs", flush=True)
    Q, K, V, dO = (p.f64(k) for k in ("Q", "K", "V", "dO"))
    t0 = time.perf_counter()
    out, lse = oracle.forward(p.indptr, p.indices, Q, K, V)
    print(f"whole-tensor case {name}: oracle forward {time.perf_counter() - t0:.1f}s", flush=True)
    assert_close("out", res.pop("out"), out, tol)
    assert_lse_close(res.pop("lse"), lse, tol)
    empty = np.diff(p.indptr) == 0
    del out, lse
    t0 = time.perf_counter()
    dQ, dK, dV = oracle.backward(p.indptr, p.indices, Q, K, V, dO)
    print(f"whole-tensor case {name}: oracle backward {time.perf_counter() - t0:.1f}s", flush=True)
    del Q, K, V, dO
    got = res.pop("dQ")
    assert np.all(got[empty] == 0.0)
    assert_close("dQ", got, dQ, tol)
    del got, dQ
    unused = np.ones(p.n_src, dtype=bool)
    unused[p.indices] = False
    for key, ref in (("dK", dK), ("dV", dV)):
        got = res.pop(key)
        assert np.all(got[unused] == 0.0)
        assert_close(key, got, ref, tol)
        del got
