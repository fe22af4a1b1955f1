"""GPU plan builder vs the numpy reference: every array bit for bit."""
import numpy as np
import pytest
import torch

import gen
from oracle import plan_ref as pr

pytestmark = pytest.mark.gpu


def build_and_compare(indptr, indices, n_src, wave_max_deg, hub_chunk):
    import paper_2604_16715_amd as gta
    d_ptr = torch.from_numpy(np.ascontiguousarray(indptr, dtype=np.int64)).cuda()
    d_idx = torch.from_numpy(np.ascontiguousarray(indices, dtype=np.int32)).cuda()
    plan = gta.gta_plan_create(d_ptr, d_idx, n_src, wave_max_deg=wave_max_deg, hub_chunk=hub_chunk,
                               validate=True)
    ref = pr.plan_ref(indptr, indices, n_src, wave_max_deg, hub_chunk)
    tr = plan.export_transpose()
    for k in ("t_indptr", "t_indices", "t_eid"):
        np.testing.assert_array_equal(tr[k], ref[k], err_msg=k)
    for side, name in ((0, "dst"), (1, "src")):
        got = plan.export_bins(side)
        want = ref[name]
        assert got["n_chunked"] == want["n_chunked"] and got["n_hub"] == want["n_hub"], name
        np.testing.assert_array_equal(got["bin_off"], want["bin_off"], err_msg=name)
        np.testing.assert_array_equal(got["bin_rows"], want["bin_rows"], err_msg=name)
        np.testing.assert_array_equal(got["chunk_ptr"].astype(np.int64), want["chunk_ptr"], err_msg=name)
        np.testing.assert_array_equal(got["chunks"], want["chunks"], err_msg=name)
    return plan


@pytest.mark.parametrize("name,shrink,wmax,chunk", [
    ("tiny", 1, 128, 2048), ("tiny", 1, 8, 32), ("mid", 1, 128, 2048), ("mid", 4, 16, 16),
    ("large", 32, 128, 2048), ("partition", 32, 64, 256), ("skew", 64, 512, 2048),
])
def test_plan_matches_reference(name, shrink, wmax, chunk):
    print(f"plan case {name} shrink={shrink} wave_max={wmax} hub_chunk={chunk}", flush=True)
    w = gen.workload(name, shrink)
    build_and_compare(w.indptr, w.indices, w.n_src, wmax, chunk)


def test_plan_edge_cases():
    # no entries at all
    build_and_compare(np.zeros(8, dtype=np.int64), np.zeros(0, dtype=np.int32), 9, 4, 8)
    # a single row holding everything, duplicates included; unsorted
    idx = np.array([5, 1, 5, 0, 3, 3, 3, 2, 7, 7, 6, 1, 0], dtype=np.int32)
    build_and_compare(np.array([0, len(idx)], dtype=np.int64), idx, 8, 2, 4)
    # unsorted rows with duplicates and empty rows, sizes crossing several 2048-key tiles
    indptr, indices = gen.random_csr(3000, 5000, 40000, seed=77, allow_dup=True, sort_rows=False)
    build_and_compare(indptr, indices, 5000, 8, 16)


def test_plan_rejects_malformed_graph():
    import paper_2604_16715_amd as gta
    indptr = torch.tensor([0, 2, 3], dtype=torch.int64).cuda()
    indices = torch.tensor([0, 9, 1], dtype=torch.int32).cuda()
    with pytest.raises(gta.GtaError) as e:
        gta.gta_plan_create(indptr, indices, 4, validate=True)
    assert e.value.status == 5
    with pytest.raises(gta.GtaError) as e:
        gta.gta_plan_create(indptr, indices, 1, validate=False)   # n_src < n_dst
    assert e.value.status == 1


def test_plan_compaction_keeps_every_array_and_result():
    """gta_plan_compact moves the plan into a buffer of the retained size: the exported arrays are those
    of the plan built in place, and attention through the moved plan (with the build workspace
    overwritten) gives the bits of the in-place one."""
    import paper_2604_16715_amd as gta
    from helpers import Problem, to_torch
    w = gen.workload("mid", 4)
    p = Problem.from_workload(w)
    d_ptr, d_idx = torch.from_numpy(w.indptr).cuda(), torch.from_numpy(w.indices).cuda()
    kw = dict(wave_max_deg=16, hub_chunk=64, keep_dz_min_nnz=1)
    in_place = gta.gta_plan_create(d_ptr, d_idx, w.n_src, compact=False, **kw)
    lib = gta.load_library()
    import ctypes
    opts = gta.binding._PlanOpts(0, kw["wave_max_deg"], kw["hub_chunk"], 1, kw["keep_dz_min_nnz"])
    keep = lib.gta_plan_retained_bytes(w.n_dst, w.n_src, w.nnz, ctypes.byref(opts))
    assert 0 < keep < in_place.workspace.numel()
    moved = gta.gta_plan_create(d_ptr, d_idx, w.n_src, compact=True, **kw)
    assert moved.workspace.numel() == max(keep, 256)
    a, b = in_place.export_transpose(), moved.export_transpose()
    for k in a:
        np.testing.assert_array_equal(a[k], b[k], err_msg=k)
    for side in (0, 1):
        a, b = in_place.export_bins(side), moved.export_bins(side)
        for k in ("bin_rows", "bin_off", "chunk_ptr", "chunks"):
            np.testing.assert_array_equal(a[k], b[k], err_msg=f"side {side} {k}")
    # compaction through the C ABI by hand, then the old buffer is filled with garbage
    third = gta.gta_plan_create(d_ptr, d_idx, w.n_src, compact=False, **kw)
    old = third.workspace
    new = torch.empty(keep, dtype=torch.uint8, device="cuda")
    rc = lib.gta_plan_compact(third.handle, new.data_ptr(), new.numel(), None)
    assert rc == 0, lib.gta_last_error().decode()
    old.fill_(0xA5)
    third.workspace = new
    assert lib.gta_plan_compact(third.handle, new.data_ptr() + 256, new.numel(), None) == 1   # overlapping target
    Q, K, V, dO = (to_torch(getattr(p, k)) for k in ("Q", "K", "V", "dO"))
    ref_out, ref_lse = gta.gta_attn_fwd(in_place, Q, K, V)
    ref_grads = gta.gta_attn_bwd(in_place, Q, K, V, ref_out, ref_lse, dO)
    for plan in (moved, third):
        out, lse = gta.gta_attn_fwd(plan, Q, K, V)
        grads = gta.gta_attn_bwd(plan, Q, K, V, out, lse, dO)
        assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse)
        for g, r in zip(grads, ref_grads):
            assert torch.equal(g, r)
    torch.cuda.synchronize()
