"""Reference of the dense projections of the layer (Eq. 3 and Eq. 5): TEST INFRASTRUCTURE ONLY.
Plain float64 matrix products (numpy's matmul is the library primitive used as the step)."""
import numpy as np


def linear(X, W, C=None, trans_w=False):
    """X W (+ C), or X W^T (+ C) when trans_w."""
    X, W = np.asarray(X, dtype=np.float64), np.asarray(W, dtype=np.float64)
    Y = X @ (W.T if trans_w else W)
    return Y if C is None else Y + np.asarray(C, dtype=np.float64)


def linear_dw(X, dY):
    """X^T dY: the gradient of sum(dY * (X W)) with respect to W."""
    return np.asarray(X, dtype=np.float64).T @ np.asarray(dY, dtype=np.float64)
