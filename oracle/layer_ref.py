"""Reference of one Sparse Graph Attention layer (Eq. 3-5) and its gradients: TEST INFRASTRUCTURE
ONLY.  Composition, in float64, of the dense reference (Eq. 3, Eq. 5) and the attention oracle."""
import numpy as np

from . import backward as attn_backward
from . import forward as attn_forward
from .dense_ref import linear, linear_dw


def layer_forward(indptr, indices, X, Wq, Wk, Wv, Wo, heads, scale=None):
    n, d = X.shape
    D = d // heads
    Q, K, V = (linear(X, W).reshape(n, heads, D) for W in (Wq, Wk, Wv))
    Y, lse = attn_forward(indptr, indices, Q, K, V, scale)
    return linear(X, Wo, Y.reshape(n, d)), dict(Q=Q, K=K, V=V, Y=Y, lse=lse)


def layer_backward(indptr, indices, X, Wq, Wk, Wv, Wo, heads, dXout, scale=None):
    n, d = X.shape
    D = d // heads
    Q, K, V = (linear(X, W).reshape(n, heads, D) for W in (Wq, Wk, Wv))
    dQ, dK, dV = attn_backward(indptr, indices, Q, K, V, np.asarray(dXout, dtype=np.float64).reshape(n, heads, D), scale)
    dQ, dK, dV = (g.reshape(n, d) for g in (dQ, dK, dV))
    dX = (linear(dXout, Wo, trans_w=True) + linear(dQ, Wq, trans_w=True) + linear(dK, Wk, trans_w=True)
          + linear(dV, Wv, trans_w=True))
    return dX, linear_dw(X, dQ), linear_dw(X, dK), linear_dw(X, dV), linear_dw(X, dXout)
