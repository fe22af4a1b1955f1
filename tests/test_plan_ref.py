"""Pins for the numpy reference of the scheduling plan: brute force in pure Python on small
graphs, closed forms of the degree classes, and coverage properties of the chunk tables."""
import numpy as np
import pytest

from oracle import plan_ref as pr


def test_degree_class_closed_form():
    deg = np.array([0, 1, 2, 3, 4, 5, 8, 9, 16, 17, 512, 513, 2048, 2049, 2**31 - 1])
    expect = np.array([0, 1, 2, 3, 3, 4, 4, 5, 5, 6, 10, 11, 12, 13, 32])
    np.testing.assert_array_equal(pr.degree_class(deg), expect)
    # class c >= 1 covers (2^(c-2), 2^(c-1)]
    for d in range(1, 5000):
        c = int(pr.degree_class(np.array([d]))[0])
        assert d <= 2 ** (c - 1) and (c == 1 or d > 2 ** (c - 2))


@pytest.mark.parametrize("seed,n_dst,n_src,nnz,wmax,chunk", [
    (1, 50, 70, 400, 4, 8), (2, 64, 64, 3000, 8, 16), (3, 10, 10, 0, 4, 4), (4, 200, 30, 1500, 2, 2),
])
def test_plan_ref_brute_force(gen, seed, n_dst, n_src, nnz, wmax, chunk):
    indptr, indices = gen.random_csr(n_dst, n_src, max(nnz, 1), seed, allow_dup=True, sort_rows=False)
    if nnz == 0:
        indptr, indices = np.zeros(n_dst + 1, dtype=np.int64), np.zeros(0, dtype=np.int32)
    plan = pr.plan_ref(indptr, indices, n_src, wmax, chunk)
    E = int(indptr[-1])
    # transpose: brute-force list of (src, stored position, dst), sorted
    triples = sorted((int(indices[e]), e, i) for i in range(n_dst)
                     for e in range(int(indptr[i]), int(indptr[i + 1])))
    assert [t[1] for t in triples] == plan["t_eid"].tolist()
    assert [t[2] for t in triples] == plan["t_indices"].tolist()
    for j in range(n_src):
        seg = [t for t in triples if t[0] == j]
        assert plan["t_indptr"][j + 1] - plan["t_indptr"][j] == len(seg)
    assert plan["t_indptr"][0] == 0 and plan["t_indptr"][-1] == E
    for side, ptr in (("dst", indptr), ("src", plan["t_indptr"])):
        b = plan[side]
        deg = np.diff(ptr)
        n = len(deg)
        # bin_rows is a permutation ordered by (class descending, row ascending)
        rows = b["bin_rows"].tolist()
        assert sorted(rows) == list(range(n))
        cls = pr.degree_class(deg)
        keys = [(-int(cls[r]), r) for r in rows]
        assert keys == sorted(keys)
        for k in range(pr.NUM_CLASSES):
            seg = rows[int(b["bin_off"][k]): int(b["bin_off"][k + 1])]
            assert all(cls[r] == pr.NUM_CLASSES - 1 - k for r in seg)
        assert b["bin_off"][-1] == n
        # chunked rows are exactly the rows above the wave threshold, as a prefix
        nch = b["n_chunked"]
        assert set(rows[:nch]) == {r for r in range(n) if deg[r] > wmax}
        assert set(rows[: b["n_hub"]]) == {r for r in range(n) if deg[r] > chunk}
        # chunks tile each chunked row's entries exactly once, in order
        c = 0
        for k, r in enumerate(rows[:nch]):
            assert b["chunk_ptr"][k] == c
            pos = int(ptr[r])
            nck = -(-int(deg[r]) // chunk)
            for s in range(nck):
                row, beg, end, cnt = b["chunks"][c]
                assert (row, beg, cnt) == (r, pos, nck)
                assert 0 < end - beg <= chunk and (end - beg == chunk or s == nck - 1)
                pos = end
                c += 1
            assert pos == ptr[r + 1]
        assert b["chunk_ptr"][nch] == c == len(b["chunks"])
