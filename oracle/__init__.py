"""CPU oracle for sparse graph attention: TEST INFRASTRUCTURE ONLY.

Importable only from tests, the smoke check and the benchmark's cpu_baseline leg.  The
arithmetic lives in ``sga_oracle.cpp`` (double precision, one function per operator of
Section 2); this module only marshals numpy arrays.  ``plan_ref`` is the numpy reference of
the integer scheduling plan.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from . import plan_ref  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
# SGA_SANITIZE=1 selects a host build with AddressSanitizer + UndefinedBehaviorSanitizer in its own
# file (run python with the ASan runtime preloaded: LD_PRELOAD=$(g++ -print-file-name=libasan.so))
_SANITIZE = os.environ.get("SGA_SANITIZE", "") == "1"
_LIB_PATH = os.path.join(_HERE, "libsga_oracle_san.so" if _SANITIZE else "libsga_oracle.so")
_CXXFLAGS = (["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
             if _SANITIZE else ["-O2"])
_lib = None


def build(force: bool = True) -> str:
    src = os.path.join(_HERE, "sga_oracle.cpp")
    if force or not os.path.exists(_LIB_PATH):
        subprocess.check_call(
            ["g++", *_CXXFLAGS, "-std=c++17", "-fopenmp", "-fPIC", "-shared", "-o", _LIB_PATH, src]
        )
    return _LIB_PATH


def _open(path):
    """A built oracle library with its prototypes set (tests also open deliberately broken builds with it)."""
    lib = ctypes.CDLL(path)
    i64, ci, dbl, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_double, ctypes.c_void_p
    lib.sga_forward.restype = ci
    lib.sga_forward.argtypes = [i64, i64, vp, vp, ci, ci, dbl, vp, vp, vp, vp, vp, vp]
    lib.sga_backward.restype = ci
    lib.sga_backward.argtypes = [i64, i64, vp, vp, ci, ci, dbl, vp, vp, vp, vp, vp, vp, vp, ci]
    return lib


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        _lib = _open(_LIB_PATH)
    return _lib


def _f64(x):
    return np.ascontiguousarray(x, dtype=np.float64)


def _graph(indptr, indices):
    return (np.ascontiguousarray(indptr, dtype=np.int64),
            np.ascontiguousarray(indices, dtype=np.int32))


def forward(indptr, indices, Q, K, V, scale=None, want_alpha=False):
    """Y [n_dst,H,D], lse [n_dst,H] (and U [E,H] when want_alpha) in float64."""
    lib = _load()
    indptr, indices = _graph(indptr, indices)
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    n_dst, H, D = Q.shape
    n_src = K.shape[0]
    assert indptr.shape[0] == n_dst + 1 and K.shape == V.shape and K.shape[1:] == (H, D)
    assert indices.shape[0] >= indptr[-1]
    if indptr[-1] > 0:
        assert 0 <= indices[:indptr[-1]].min() and indices[:indptr[-1]].max() < n_src
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    Y = np.empty((n_dst, H, D), dtype=np.float64)
    lse = np.empty((n_dst, H), dtype=np.float64)
    U = np.empty((int(indptr[-1]), H), dtype=np.float64) if want_alpha else None
    lib.sga_forward(n_dst, n_src, indptr.ctypes.data, indices.ctypes.data, H, D, float(scale),
                    Q.ctypes.data, K.ctypes.data, V.ctypes.data, Y.ctypes.data, lse.ctypes.data,
                    U.ctypes.data if want_alpha else None)
    return (Y, lse, U) if want_alpha else (Y, lse)


def backward(indptr, indices, Q, K, V, dY, scale=None, grouped=True):
    """dQ [n_dst,H,D], dK, dV [n_src,H,D] in float64 for the loss sum(dY * Y)."""
    lib = _load()
    indptr, indices = _graph(indptr, indices)
    Q, K, V, dY = _f64(Q), _f64(K), _f64(V), _f64(dY)
    n_dst, H, D = Q.shape
    n_src = K.shape[0]
    assert dY.shape == Q.shape and K.shape == V.shape and indptr.shape[0] == n_dst + 1
    if indptr[-1] > 0:
        assert 0 <= indices[:indptr[-1]].min() and indices[:indptr[-1]].max() < n_src
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    dQ = np.empty_like(Q)
    dK = np.empty_like(K)
    dV = np.empty_like(V)
    lib.sga_backward(n_dst, n_src, indptr.ctypes.data, indices.ctypes.data, H, D, float(scale),
                     Q.ctypes.data, K.ctypes.data, V.ctypes.data, dY.ctypes.data,
                     dQ.ctypes.data, dK.ctypes.data, dV.ctypes.data, int(bool(grouped)))
    return dQ, dK, dV


# ---- the individual operators (same functions forward() / backward() are composed of) -------
def _op_protos(lib):
    i64, ci, dbl, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_double, ctypes.c_void_p
    lib.sga_sddmm.restype = None
    lib.sga_sddmm.argtypes = [i64, vp, vp, ci, ci, vp, vp, vp]
    lib.sga_edge_softmax.restype = None
    lib.sga_edge_softmax.argtypes = [i64, vp, ci, dbl, vp, vp, vp]
    lib.sga_edge_softmax_bwd.restype = None
    lib.sga_edge_softmax_bwd.argtypes = [i64, vp, ci, dbl, vp, vp, vp]
    lib.sga_spmm.restype = None
    lib.sga_spmm.argtypes = [i64, vp, vp, ci, ci, vp, vp, vp]
    lib.sga_spmm_t.restype = None
    lib.sga_spmm_t.argtypes = [i64, i64, vp, vp, ci, ci, vp, vp, vp]
    return lib


def sddmm(indptr, indices, X, Y):
    """Z [E,H]: per stored entry (i <- j) and head, the dot product of X[i,h] and Y[j,h]."""
    lib = _op_protos(_load())
    indptr, indices = _graph(indptr, indices)
    X, Y = _f64(X), _f64(Y)
    n_dst, H, D = X.shape
    Z = np.empty((int(indptr[-1]), H), dtype=np.float64)
    lib.sga_sddmm(n_dst, indptr.ctypes.data, indices.ctypes.data, H, D, X.ctypes.data, Y.ctypes.data, Z.ctypes.data)
    return Z


def edge_softmax(indptr, Z, scale):
    lib = _op_protos(_load())
    indptr = np.ascontiguousarray(indptr, dtype=np.int64)
    Z = _f64(Z)
    n_dst, H = indptr.shape[0] - 1, Z.shape[1]
    U = np.zeros_like(Z)
    lse = np.empty((n_dst, H), dtype=np.float64)
    lib.sga_edge_softmax(n_dst, indptr.ctypes.data, H, float(scale), Z.ctypes.data, U.ctypes.data, lse.ctypes.data)
    return U, lse


def edge_softmax_bwd(indptr, U, dU, scale):
    lib = _op_protos(_load())
    indptr = np.ascontiguousarray(indptr, dtype=np.int64)
    U, dU = _f64(U), _f64(dU)
    dZ = np.zeros_like(U)
    lib.sga_edge_softmax_bwd(indptr.shape[0] - 1, indptr.ctypes.data, U.shape[1], float(scale), U.ctypes.data,
                             dU.ctypes.data, dZ.ctypes.data)
    return dZ


def spmm(indptr, indices, W, X, n_src=None, transposed=False):
    """transposed=False: Y[i] = sum_e W[e] X[j];  transposed=True: Y[j] = sum_e W[e] X[i] (serial scatter)."""
    lib = _op_protos(_load())
    indptr, indices = _graph(indptr, indices)
    W, X = _f64(W), _f64(X)
    n_dst = indptr.shape[0] - 1
    _, H, D = X.shape
    if not transposed:
        Y = np.empty((n_dst, H, D), dtype=np.float64)
        lib.sga_spmm(n_dst, indptr.ctypes.data, indices.ctypes.data, H, D, W.ctypes.data, X.ctypes.data, Y.ctypes.data)
    else:
        Y = np.empty((n_src, H, D), dtype=np.float64)
        lib.sga_spmm_t(n_dst, n_src, indptr.ctypes.data, indices.ctypes.data, H, D, W.ctypes.data, X.ctypes.data,
                       Y.ctypes.data)
    return Y


def merge(out_a, lse_a, out_b, lse_b):
    """Attention over the union of two disjoint sets of stored entries of the same rows, from the
    two partial results (out [n,H,D], lse [n,H]): the softmax denominators add,
    lse = log(exp(lse_a) + exp(lse_b)), and each partial output is re-weighted by its share
    exp(lse_x - lse) of the total (Eq. 2 with the neighbour sum split in two).  A side whose lse is
    -inf (no entries) contributes nothing; both -inf gives out = 0, lse = -inf.  float64."""
    out_a, out_b = _f64(out_a), _f64(out_b)
    lse_a, lse_b = _f64(lse_a), _f64(lse_b)
    with np.errstate(divide="ignore", invalid="ignore"):
        lse = np.logaddexp(lse_a, lse_b)
        wa = np.where(np.isneginf(lse_a), 0.0, np.exp(lse_a - lse))
        wb = np.where(np.isneginf(lse_b), 0.0, np.exp(lse_b - lse))
    wa = np.nan_to_num(wa, nan=0.0)
    wb = np.nan_to_num(wb, nan=0.0)
    return wa[..., None] * out_a + wb[..., None] * out_b, lse
