"""GPU forward/backward vs the fp64 oracle, element by element, through the C ABI."""
import numpy as np
import pytest
import torch

import gen
from helpers import TOL, Problem, assert_close, assert_lse_close, run_gpu

pytestmark = pytest.mark.gpu


def check(p: Problem, scale=0.0, plan_kwargs=None, tag=""):
    print(f"attn case {tag} n_dst={p.n_dst} n_src={p.n_src} nnz={int(p.indptr[-1])} "
          f"shape={p.Q.shape[1:]} dtype={p.dtype} plan={plan_kwargs}", flush=True)
    tol = TOL[p.dtype]
    o_scale = None if scale <= 0 else scale
    out, lse = p.oracle_forward(o_scale)
    dQ, dK, dV = p.oracle_backward(o_scale)
    empty = np.diff(p.indptr) == 0
    unused = np.ones(p.n_src, dtype=bool)
    unused[p.indices] = False
    # both backward forms: dZ kept per stored entry (recommended scratch) and nothing kept (minimum scratch)
    for lean in (False, True):
        res = run_gpu(p, scale, plan_kwargs, lean_scratch=lean)
        assert_close("out", res["out"], out, tol)
        assert_lse_close(res["lse"], lse, tol)
        assert np.all(res["out"][empty] == 0.0) and np.all(res["dQ"][empty] == 0.0)
        assert_close("dQ", res["dQ"], dQ, tol)
        assert_close("dK", res["dK"], dK, tol)
        assert_close("dV", res["dV"], dV, tol)
        assert np.all(res["dK"][unused] == 0.0) and np.all(res["dV"][unused] == 0.0)
    return res


# the five benchmark workloads, at sizes the oracle finishes in seconds (the first two in full)
@pytest.mark.parametrize("name,shrink", [("tiny", 1), ("mid", 1), ("large", 16), ("partition", 16), ("skew", 32)])
def test_workloads_default_plan(name, shrink):
    check(Problem.from_workload(gen.workload(name, shrink)), tag=f"{name}/{shrink}")


# small thresholds push many rows through the chunk + merge kernels
@pytest.mark.parametrize("name,shrink,kw", [
    ("tiny", 1, dict(wave_max_deg=8, hub_chunk=32)),
    ("tiny", 1, dict(wave_max_deg=64, hub_chunk=64, pack_max_deg=2)),
    ("mid", 8, dict(wave_max_deg=16, hub_chunk=128, pack_max_deg=16)),
    ("large", 64, dict(wave_max_deg=32, hub_chunk=256)),
    ("skew", 128, dict(wave_max_deg=4, hub_chunk=4, pack_max_deg=1)),
])
def test_workloads_forced_schedules(name, shrink, kw):
    check(Problem.from_workload(gen.workload(name, shrink)), plan_kwargs=kw, tag=f"{name}/{shrink}")


# every supported (heads, head_dim, dtype) geometry class on a ragged random graph
@pytest.mark.parametrize("heads,head_dim,dtype", [
    (4, 8, "f32"), (2, 16, "f32"), (8, 8, "f32"), (1, 32, "f32"), (4, 64, "f32"), (16, 16, "f32"),
    (1, 64, "f32"), (2, 64, "f32"), (8, 32, "f32"),
    (4, 16, "bf16"), (8, 16, "bf16"), (2, 32, "bf16"), (1, 64, "bf16"), (4, 128, "bf16"),
    (16, 32, "bf16"), (2, 128, "bf16"), (8, 64, "bf16"), (32, 16, "bf16"),
    # one 16-byte lane per head, and 64-byte rows (4 lanes)
    (8, 8, "bf16"), (16, 4, "f32"), (64, 8, "bf16"), (4, 4, "f32"), (2, 16, "bf16"), (1, 16, "f32"),
    # rows wider than 1024 bytes and head counts that are not powers of two: several slices per row
    (8, 64, "f32"), (16, 64, "bf16"), (3, 16, "f32"), (12, 16, "bf16"), (6, 32, "bf16"), (5, 64, "f32"),
])
def test_geometries(heads, head_dim, dtype):
    indptr, indices = gen.random_csr(700, 900, 9000, seed=heads * 1000 + head_dim, allow_dup=True, sort_rows=False)
    # plant a few long rows so every schedule runs
    deg = np.diff(indptr)
    p = Problem.random(indptr, indices, 900, heads, head_dim, dtype, seed=heads + head_dim)
    check(p, plan_kwargs=dict(wave_max_deg=16, hub_chunk=32), tag=f"geom {heads}x{head_dim} {dtype}")


def test_edge_cases():
    # empty graph: all outputs zero, lse -inf
    p = Problem.random(np.zeros(6, dtype=np.int64), np.zeros(0, dtype=np.int32), 7, 4, 16, "f32", 1)
    res = check(p, tag="empty")
    assert np.all(res["dK"] == 0) and np.all(np.isneginf(res["lse"]))
    # one row holding 5000 entries (hub split + merge), sources repeated
    rng = np.random.Generator(np.random.Philox(5))
    idx = rng.integers(0, 50, size=5000).astype(np.int32)
    p = Problem.random(np.array([0, 5000], dtype=np.int64), idx, 50, 8, 16, "f32", 2)
    check(p, tag="single hub row")
    # the same kind of row, short enough to be summed by a single wavefront when the thresholds allow
    p = Problem.random(np.array([0, 1800], dtype=np.int64), idx[:1800], 50, 8, 16, "f32", 2)
    check(p, plan_kwargs=dict(wave_max_deg=2048, hub_chunk=2048), tag="long row, one wavefront")
    # one source attended by every row (hub on the transposed side); explicit scale
    n = 3000
    p = Problem.random(np.arange(n + 1, dtype=np.int64), np.zeros(n, dtype=np.int32), 1 + n, 4, 16, "bf16", 3)
    check(p, scale=0.4, tag="single hub source")
    # large scores must not overflow
    indptr, indices = gen.random_csr(64, 64, 700, seed=9)
    p = Problem.random(indptr, indices, 64, 4, 16, "f32", 4)
    p.Q = (p.Q * 60.0).astype(np.float32)
    check(p, tag="large scores")


def test_bitwise_reproducible():
    w = gen.workload("mid", 8)
    p = Problem.from_workload(w)
    kw = dict(wave_max_deg=16, hub_chunk=64)
    for lean in (False, True):
        a = run_gpu(p, plan_kwargs=kw, lean_scratch=lean)
        b = run_gpu(p, plan_kwargs=kw, lean_scratch=lean)
        for k in ("out", "lse", "dQ", "dK", "dV"):
            assert np.array_equal(a[k], b[k], equal_nan=True), k


def test_unsupported_shapes_are_reported():
    import paper_2604_16715_amd as gta
    indptr, indices = gen.random_csr(16, 16, 40, seed=3)
    plan = gta.gta_plan_create(torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda(), 16)
    for heads, head_dim, dt in ((4, 12, torch.float32), (2, 4, torch.bfloat16), (1, 8, torch.bfloat16),
                                (6, 8, torch.bfloat16)):
        q = torch.zeros((16, heads, head_dim), dtype=dt, device="cuda")
        with pytest.raises(gta.GtaError) as e:
            gta.gta_attn_fwd(plan, q, q, q)
        assert e.value.status == 2
    q = torch.zeros((16, 4, 16), dtype=torch.float16, device="cuda")
    with pytest.raises(gta.GtaError):
        gta.gta_attn_fwd(plan, q, q, q)
