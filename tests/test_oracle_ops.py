"""The oracle's individual operators against plain numpy definitions (CPU only)."""
import numpy as np

import gen
import oracle


def test_operator_functions_match_numpy_definitions():
    n_dst, n_src, H, D = 40, 55, 2, 3
    indptr, indices = gen.random_csr(n_dst, n_src, 300, seed=5, allow_dup=True, sort_rows=False)
    E = int(indptr[-1])
    rng = np.random.Generator(np.random.Philox(6))
    X, Y = rng.standard_normal((n_dst, H, D)), rng.standard_normal((n_src, H, D))
    dst = np.repeat(np.arange(n_dst), np.diff(indptr))
    Z = oracle.sddmm(indptr, indices, X, Y)
    np.testing.assert_allclose(Z, np.einsum("ehd,ehd->eh", X[dst], Y[indices]), rtol=1e-13, atol=1e-14)
    scale = 0.7
    U, lse = oracle.edge_softmax(indptr, Z, scale)
    for i in range(n_dst):
        seg = slice(int(indptr[i]), int(indptr[i + 1]))
        if seg.start == seg.stop:
            assert np.all(np.isneginf(lse[i]))
            continue
        ex = np.exp(scale * Z[seg])
        np.testing.assert_allclose(U[seg], ex / ex.sum(axis=0), rtol=1e-12)
        np.testing.assert_allclose(lse[i], np.log(ex.sum(axis=0)), rtol=1e-12, atol=1e-13)
    W = rng.standard_normal((E, H))
    ref = np.zeros((n_dst, H, D))
    np.add.at(ref, dst, W[:, :, None] * Y[indices])
    np.testing.assert_allclose(oracle.spmm(indptr, indices, W, Y), ref, rtol=1e-12, atol=1e-13)
    ref_t = np.zeros((n_src, H, D))
    np.add.at(ref_t, indices, W[:, :, None] * X[dst])
    np.testing.assert_allclose(oracle.spmm(indptr, indices, W, X, n_src, transposed=True), ref_t, rtol=1e-12, atol=1e-13)
    dU = rng.standard_normal((E, H))
    dZ = oracle.edge_softmax_bwd(indptr, U, dU, scale)
    rowdot = np.zeros((n_dst, H))
    np.add.at(rowdot, dst, U * dU)
    np.testing.assert_allclose(dZ, scale * U * (dU - rowdot[dst]), rtol=1e-12, atol=1e-14)


def split_graph(indptr, indices, keep):
    """Two CSR graphs over the same rows: the entries where keep is True, and the others."""
    n = len(indptr) - 1
    dst = np.repeat(np.arange(n), np.diff(indptr))
    parts = []
    for mask in (keep, ~keep):
        cnt = np.bincount(dst[mask], minlength=n)
        parts.append((np.concatenate([[0], np.cumsum(cnt)]).astype(np.int64), indices[mask].astype(np.int32)))
    return parts


def test_merge_of_two_entry_sets_is_attention_over_their_union():
    # pins oracle.merge AND the forward's lse: attention over a split neighbourhood, merged, must be
    # the attention over the whole neighbourhood (Eq. 2 with the sum over N(i) cut in two)
    n_dst, n_src, H, D = 60, 80, 3, 4
    indptr, indices = gen.random_csr(n_dst, n_src, 700, seed=11, allow_dup=True, sort_rows=False)
    rng = np.random.Generator(np.random.Philox(12))
    Q = rng.standard_normal((n_dst, H, D))
    K, V = rng.standard_normal((n_src, H, D)), rng.standard_normal((n_src, H, D))
    full_out, full_lse = oracle.forward(indptr, indices, Q, K, V)
    for keep in (indices < 30, rng.random(len(indices)) < 0.5, np.zeros(len(indices), dtype=bool)):
        (pa, ia), (pb, ib) = split_graph(indptr, indices, keep)
        oa, la = oracle.forward(pa, ia, Q, K, V)
        ob, lb = oracle.forward(pb, ib, Q, K, V)
        out, lse = oracle.merge(oa, la, ob, lb)
        np.testing.assert_allclose(out, full_out, rtol=1e-12, atol=1e-13)
        assert np.array_equal(np.isneginf(lse), np.isneginf(full_lse))
        fin = np.isfinite(full_lse)
        np.testing.assert_allclose(lse[fin], full_lse[fin], rtol=1e-12, atol=1e-13)
    # closed form: two single-entry sides with scores s_a, s_b give weights sigmoid(s_a - s_b)
    oa, ob = np.array([[[1.0, 0.0]]]), np.array([[[0.0, 1.0]]])
    out, lse = oracle.merge(oa, np.array([[0.3]]), ob, np.array([[-0.9]]))
    w = 1.0 / (1.0 + np.exp(-1.2))
    np.testing.assert_allclose(out, [[[w, 1.0 - w]]], rtol=1e-14)
    np.testing.assert_allclose(lse, [[np.log(np.exp(0.3) + np.exp(-0.9))]], rtol=1e-14)
