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
