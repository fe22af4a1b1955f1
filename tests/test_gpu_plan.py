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
