"""Pins of the dense reference: explicit loops on tiny inputs and a finite-difference check that
linear_dw is the weight gradient of linear (CPU only)."""
import numpy as np

from oracle import dense_ref


def test_linear_matches_explicit_loops():
    rng = np.random.Generator(np.random.Philox(1))
    X, W, C = rng.standard_normal((5, 4)), rng.standard_normal((4, 3)), rng.standard_normal((5, 3))
    want = np.zeros((5, 3))
    for r in range(5):
        for o in range(3):
            want[r, o] = sum(X[r, k] * W[k, o] for k in range(4)) + C[r, o]
    np.testing.assert_allclose(dense_ref.linear(X, W, C), want, rtol=1e-14)
    np.testing.assert_allclose(dense_ref.linear(X, W.T.copy(), C, trans_w=True), want, rtol=1e-14)
    dY = rng.standard_normal((5, 3))
    want_dw = np.zeros((4, 3))
    for k in range(4):
        for o in range(3):
            want_dw[k, o] = sum(X[r, k] * dY[r, o] for r in range(5))
    np.testing.assert_allclose(dense_ref.linear_dw(X, dY), want_dw, rtol=1e-14)
    # weight gradient by central differences of L = sum(dY * (X W))
    num = np.zeros_like(W)
    for k in range(4):
        for o in range(3):
            Wp, Wm = W.copy(), W.copy()
            Wp[k, o] += 1e-6
            Wm[k, o] -= 1e-6
            num[k, o] = (np.sum(dY * dense_ref.linear(X, Wp)) - np.sum(dY * dense_ref.linear(X, Wm))) / 2e-6
    np.testing.assert_allclose(num, want_dw, rtol=1e-8, atol=1e-9)


def test_layer_reference_gradients_match_finite_differences():
    import gen
    from oracle import layer_ref
    n, heads, D = 9, 2, 3
    d = heads * D
    indptr, indices = gen.random_csr(n, n, 30, seed=4)
    rng = np.random.Generator(np.random.Philox(8))
    X = rng.standard_normal((n, d))
    Ws = [0.4 * rng.standard_normal((d, d)) for _ in range(4)]
    dXout = rng.standard_normal((n, d))
    grads = layer_ref.layer_backward(indptr, indices, X, *Ws, heads, dXout)

    def loss(Xv, Wv):
        return float(np.sum(dXout * layer_ref.layer_forward(indptr, indices, Xv, *Wv, heads)[0]))

    h = 1e-6
    params = [X] + Ws            # gradient order returned: dX, dWq, dWk, dWv, dWo
    for which, G in enumerate(grads):
        num = np.zeros_like(params[which])
        for idx in np.ndindex(*params[which].shape):
            hi = [p.copy() for p in params]
            lo = [p.copy() for p in params]
            hi[which][idx] += h
            lo[which][idx] -= h
            num[idx] = (loss(hi[0], hi[1:]) - loss(lo[0], lo[1:])) / (2 * h)
        assert np.max(np.abs(num - G)) <= 1e-6 * max(1.0, np.max(np.abs(G))), which
