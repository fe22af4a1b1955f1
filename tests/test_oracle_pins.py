"""Pins for the CPU oracle: everything here checks oracle/ against something that is not
the oracle — a hand-worked example, dense brute force with multiplicities, a library routine
on the complete graph, closed forms, invariants, finite differences and autograd of a dense
formulation.  CPU only."""
import json
import os

import numpy as np
import pytest
import torch

HERE = os.path.dirname(os.path.abspath(__file__))


# --------------------------------------------------------------------------- helpers
def dense_attention(indptr, indices, Q, K, V, scale):
    """Dense masked softmax attention with entry multiplicities, numpy float64.
    Row i attends to source j with weight C[i,j]*exp(scale*q_i.k_j) / sum_j(...)."""
    n_dst, H, D = Q.shape
    n_src = K.shape[0]
    dst = np.repeat(np.arange(n_dst), np.diff(indptr))
    C = np.zeros((n_dst, n_src))
    np.add.at(C, (dst, indices[: indptr[-1]]), 1.0)
    S = scale * np.einsum("ihd,jhd->hij", Q, K)
    Smask = np.where(C[None] > 0, S, -np.inf)
    m = Smask.max(axis=2, keepdims=True)
    m = np.where(np.isfinite(m), m, 0.0)
    W = C[None] * np.exp(np.where(C[None] > 0, S - m, -np.inf))
    den = W.sum(axis=2, keepdims=True)
    P = np.divide(W, den, out=np.zeros_like(W), where=den > 0)
    out = np.einsum("hij,jhd->ihd", P, V)
    with np.errstate(divide="ignore"):
        lse = (m + np.log(den))[:, :, 0].T
    return out, lse, P


def dense_attention_torch(indptr, indices, Q, K, V, scale):
    """Same thing in torch float64 so autograd can differentiate it."""
    n_dst = Q.shape[0]
    n_src = K.shape[0]
    dst = np.repeat(np.arange(n_dst), np.diff(indptr))
    C = torch.zeros((n_dst, n_src), dtype=torch.float64)
    C.index_put_((torch.as_tensor(dst), torch.as_tensor(indices[: indptr[-1]].astype(np.int64))),
                 torch.ones(len(dst), dtype=torch.float64), accumulate=True)
    S = scale * torch.einsum("ihd,jhd->hij", Q, K)
    m = torch.where(C[None] > 0, S, torch.full_like(S, -1e300)).max(dim=2, keepdim=True).values
    W = C[None] * torch.exp(torch.clamp(S - m.detach(), max=0.0) * (C[None] > 0))
    W = W * (C[None] > 0)
    den = W.sum(dim=2, keepdim=True)
    P = W / torch.where(den > 0, den, torch.ones_like(den))
    return torch.einsum("hij,jhd->ihd", P, V)


def rand_problem(gen, n_dst, n_src, nnz, H, D, seed, allow_dup=False, sort_rows=True):
    indptr, indices = gen.random_csr(n_dst, n_src, nnz, seed, allow_dup, sort_rows)
    rng = np.random.Generator(np.random.Philox(seed + 1000))
    Q = rng.standard_normal((n_dst, H, D))
    K = rng.standard_normal((n_src, H, D))
    V = rng.standard_normal((n_src, H, D))
    dO = rng.standard_normal((n_dst, H, D))
    return indptr, indices, Q, K, V, dO


# --------------------------------------------------------------------------- hand example
def test_hand_worked_example(oracle):
    g = json.load(open(os.path.join(HERE, "golden", "hand_example.json")))
    arr = lambda k: np.array(g[k], dtype=np.float64)
    indptr, indices = np.array(g["indptr"]), np.array(g["indices"], dtype=np.int32)
    out, lse, U = oracle.forward(indptr, indices, arr("Q"), arr("K"), arr("V"), g["scale"],
                                 want_alpha=True)
    np.testing.assert_allclose(out, arr("out"), rtol=0, atol=1e-14)
    np.testing.assert_allclose(U, arr("alpha"), rtol=0, atol=1e-15)
    lse_ref = np.array([[float(x) for x in row] for row in g["lse"]])
    assert lse[2, 0] == -np.inf
    np.testing.assert_allclose(lse[:2], lse_ref[:2], rtol=0, atol=1e-15)
    for grouped in (False, True):
        dQ, dK, dV = oracle.backward(indptr, indices, arr("Q"), arr("K"), arr("V"), arr("dO"),
                                     g["scale"], grouped=grouped)
        np.testing.assert_allclose(dQ, arr("dQ"), rtol=0, atol=1e-14)
        np.testing.assert_allclose(dK, arr("dK"), rtol=0, atol=1e-14)
        np.testing.assert_allclose(dV, arr("dV"), rtol=0, atol=1e-14)


# --------------------------------------------------------------------------- forward pins
@pytest.mark.parametrize("case", [
    dict(n_dst=40, n_src=40, nnz=300, H=2, D=4, seed=1),
    dict(n_dst=33, n_src=57, nnz=500, H=3, D=5, seed=2),                      # halo: n_src > n_dst
    dict(n_dst=64, n_src=64, nnz=900, H=1, D=8, seed=3, allow_dup=True),      # multiplicities
    dict(n_dst=50, n_src=20, nnz=400, H=4, D=2, seed=4, allow_dup=True, sort_rows=False),
    dict(n_dst=30, n_src=30, nnz=20, H=2, D=3, seed=5),                       # many empty rows
])
def test_forward_matches_dense_brute_force(oracle, gen, case):
    case = dict(case)
    indptr, indices, Q, K, V, _ = rand_problem(gen, **case)
    scale = 1.0 / np.sqrt(case["D"])
    out, lse, U = oracle.forward(indptr, indices, Q, K, V, scale, want_alpha=True)
    out_ref, lse_ref, P = dense_attention(indptr, indices, Q, K, V, scale)
    np.testing.assert_allclose(out, out_ref, rtol=1e-12, atol=1e-13)
    empty = np.diff(indptr) == 0
    assert np.all(out[empty] == 0.0) and np.all(lse[empty] == -np.inf)
    np.testing.assert_allclose(lse[~empty], lse_ref[~empty], rtol=1e-13, atol=1e-13)
    # per-entry weights: sum of the weights of the entries that hit (i,j) equals P[h,i,j]
    dst = np.repeat(np.arange(case["n_dst"]), np.diff(indptr))
    acc = np.zeros_like(P)
    for h in range(case["H"]):
        np.add.at(acc[h], (dst, indices), U[:, h])
    np.testing.assert_allclose(acc, P, rtol=1e-12, atol=1e-14)
    # every non-empty (row, head) sums to one
    rowsum = np.zeros((case["n_dst"], case["H"]))
    np.add.at(rowsum, dst, U)
    np.testing.assert_allclose(rowsum[~empty], 1.0, rtol=0, atol=1e-13)


def test_complete_graph_is_textbook_attention(oracle):
    n, H, D = 37, 3, 8
    rng = np.random.Generator(np.random.Philox(11))
    Q, K, V = (rng.standard_normal((n, H, D)) for _ in range(3))
    indptr = np.arange(n + 1, dtype=np.int64) * n
    indices = np.tile(np.arange(n, dtype=np.int32), n)
    out, lse = oracle.forward(indptr, indices, Q, K, V)   # default scale = 1/sqrt(D)
    tq, tk, tv = (torch.from_numpy(x).permute(1, 0, 2) for x in (Q, K, V))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).permute(1, 0, 2).numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    ref_lse = torch.logsumexp(torch.einsum("hid,hjd->hij", tq, tk) / np.sqrt(D), dim=2).T.numpy()
    np.testing.assert_allclose(lse, ref_lse, rtol=1e-13, atol=1e-13)


def test_closed_forms(oracle, gen):
    indptr, indices, Q, K, V, _ = rand_problem(gen, 60, 45, 500, 2, 4, seed=21)
    deg = np.diff(indptr)
    dst = np.repeat(np.arange(60), deg)
    nonempty = deg > 0
    # Q = 0: uniform weights -> neighbour mean, lse = ln(deg)
    out, lse = oracle.forward(indptr, indices, np.zeros_like(Q), K, V)
    mean = np.zeros_like(out)
    np.add.at(mean, dst, V[indices])
    mean[nonempty] /= deg[nonempty, None, None]
    np.testing.assert_allclose(out, mean, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(lse[nonempty], np.log(deg[nonempty])[:, None] * np.ones((1, 2)),
                               rtol=1e-14, atol=0)
    # all K rows equal: uniform weights again, lse = scale*q.k + ln(deg)
    Kc = np.broadcast_to(K[:1], K.shape).copy()
    out2, lse2 = oracle.forward(indptr, indices, Q, Kc, V)
    np.testing.assert_allclose(out2, mean, rtol=1e-12, atol=1e-13)
    s = np.einsum("ihd,hd->ih", Q, K[0]) / np.sqrt(4)
    np.testing.assert_allclose(lse2[nonempty], (s + np.log(np.maximum(deg, 1))[:, None])[nonempty],
                               rtol=1e-13, atol=1e-13)
    # rows with one entry copy the value row and lse is the score itself
    ip1 = np.arange(46, dtype=np.int64)
    ix1 = np.random.Generator(np.random.Philox(5)).permutation(45).astype(np.int32)
    Q1 = Q[:45]
    out3, lse3 = oracle.forward(ip1, ix1, Q1, K, V)
    np.testing.assert_allclose(out3, V[ix1], rtol=0, atol=1e-15)
    np.testing.assert_allclose(lse3, np.einsum("ihd,ihd->ih", Q1, K[ix1]) / 2.0, rtol=1e-14, atol=1e-15)


def test_forward_invariances(oracle, gen):
    n_dst, n_src, H, D = 48, 48, 2, 4
    indptr, indices, Q, K, V, _ = rand_problem(gen, n_dst, n_src, 400, H, D, seed=31)
    out, lse = oracle.forward(indptr, indices, Q, K, V)
    nonempty = np.diff(indptr) > 0
    # shift all K rows by c: out unchanged, lse shifts by scale * q.c
    c = np.random.Generator(np.random.Philox(32)).standard_normal((H, D))
    out_s, lse_s = oracle.forward(indptr, indices, Q, K + c[None], V)
    np.testing.assert_allclose(out_s, out, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(lse_s[nonempty], (lse + np.einsum("ihd,hd->ih", Q, c) / np.sqrt(D))[nonempty],
                               rtol=1e-12, atol=1e-12)
    # linear in V
    out_l, _ = oracle.forward(indptr, indices, Q, K, 2.5 * V + 1.0)
    np.testing.assert_allclose(out_l[nonempty], (2.5 * out + 1.0)[nonempty], rtol=1e-12, atol=1e-12)
    # explicit scale argument is honoured
    out_sc, _ = oracle.forward(indptr, indices, Q, K, V, scale=0.37)
    ref_sc, _, _ = dense_attention(indptr, indices, Q, K, V, 0.37)
    np.testing.assert_allclose(out_sc, ref_sc, rtol=1e-12, atol=1e-13)
    # relabelling nodes (same permutation on both sides) permutes the result
    perm = np.random.Generator(np.random.Philox(33)).permutation(n_dst)   # new id of old node
    inv = np.argsort(perm)
    dst = np.repeat(np.arange(n_dst), np.diff(indptr))
    nd, ns = perm[dst], perm[indices]
    order = np.lexsort((ns, nd))
    ip2 = np.zeros(n_dst + 1, dtype=np.int64)
    np.add.at(ip2, nd + 1, 1)
    ip2 = np.cumsum(ip2)
    out_p, lse_p = oracle.forward(ip2, ns[order].astype(np.int32), Q[inv], K[inv], V[inv])
    np.testing.assert_allclose(out_p[perm], out, rtol=1e-12, atol=1e-13)
    np.testing.assert_array_equal(np.isinf(lse_p[perm]), np.isinf(lse))
    np.testing.assert_allclose(lse_p[perm][nonempty], lse[nonempty], rtol=1e-13, atol=1e-13)


def test_large_scores_are_stable(oracle, gen):
    indptr, indices, Q, K, V, _ = rand_problem(gen, 20, 20, 120, 1, 4, seed=41)
    out, lse = oracle.forward(indptr, indices, 3000.0 * Q, K, V)
    assert np.all(np.isfinite(out))
    ref, _, _ = dense_attention(indptr, indices, 3000.0 * Q, K, V, 0.5)
    np.testing.assert_allclose(out, ref, rtol=1e-10, atol=1e-12)


# --------------------------------------------------------------------------- backward pins
@pytest.mark.parametrize("case", [
    dict(n_dst=24, n_src=24, nnz=120, H=2, D=3, seed=51),
    dict(n_dst=17, n_src=29, nnz=150, H=1, D=4, seed=52, allow_dup=True, sort_rows=False),
    dict(n_dst=20, n_src=20, nnz=15, H=2, D=2, seed=53),
])
def test_backward_matches_autograd_of_dense_form(oracle, gen, case):
    indptr, indices, Q, K, V, dO = rand_problem(gen, **case)
    scale = 1.0 / np.sqrt(case["D"])
    tq, tk, tv = (torch.tensor(x, requires_grad=True) for x in (Q, K, V))
    y = dense_attention_torch(indptr, indices, tq, tk, tv, scale)
    (y * torch.from_numpy(dO)).sum().backward()
    for grouped in (False, True):
        dQ, dK, dV = oracle.backward(indptr, indices, Q, K, V, dO, scale, grouped=grouped)
        np.testing.assert_allclose(dQ, tq.grad.numpy(), rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(dK, tk.grad.numpy(), rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(dV, tv.grad.numpy(), rtol=1e-11, atol=1e-12)


def test_backward_matches_finite_differences(oracle, gen):
    indptr, indices, Q, K, V, dO = rand_problem(gen, 10, 13, 45, 2, 3, seed=61)
    scale = 0.61
    dQ, dK, dV = oracle.backward(indptr, indices, Q, K, V, dO, scale, grouped=False)

    def loss(q, k, v):
        return float(np.sum(dO * oracle.forward(indptr, indices, q, k, v, scale)[0]))

    h = 1e-5
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        num = np.zeros_like(X)
        it = np.nditer(X, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            Xp, Xm = X.copy(), X.copy()
            Xp[idx] += h
            Xm[idx] -= h
            args_p = dict(Q=Q, K=K, V=V)
            args_m = dict(Q=Q, K=K, V=V)
            args_p[name], args_m[name] = Xp, Xm
            num[idx] = (loss(args_p["Q"], args_p["K"], args_p["V"]) -
                        loss(args_m["Q"], args_m["K"], args_m["V"])) / (2 * h)
        err = np.max(np.abs(num - G)) / max(1e-30, np.max(np.abs(G)))
        assert err < 1e-6, (name, err)


def test_backward_invariants(oracle, gen):
    n_dst, n_src, H, D = 70, 90, 3, 4
    indptr, indices, Q, K, V, dO = rand_problem(gen, n_dst, n_src, 160, H, D, seed=71)
    dQ, dK, dV = oracle.backward(indptr, indices, Q, K, V, dO)
    dQs, dKs, dVs = oracle.backward(indptr, indices, Q, K, V, dO, grouped=False)
    for a, b in ((dQ, dQs), (dK, dKs), (dV, dVs)):
        np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-14)
    nonempty = np.diff(indptr) > 0
    # weights of a row sum to one => the value gradients add up to the output gradients
    np.testing.assert_allclose(dV.sum(axis=0), dO[nonempty].sum(axis=0), rtol=1e-12, atol=1e-12)
    # scores are bilinear in (q, k): sum_i q_i.dQ_i == sum_j k_j.dK_j per head
    np.testing.assert_allclose(np.einsum("ihd,ihd->h", Q, dQ), np.einsum("jhd,jhd->h", K, dK),
                               rtol=1e-11, atol=1e-12)
    assert np.all(dQ[~nonempty] == 0.0)
    # sources nobody attends to get no gradient
    unused = np.ones(n_src, dtype=bool)
    unused[indices] = False
    assert unused.any() and np.all(dK[unused] == 0.0) and np.all(dV[unused] == 0.0)
    # single-entry rows: softmax is constant => no dQ / dK; dV just copies dO
    ip1 = np.arange(n_dst + 1, dtype=np.int64)
    ix1 = (np.arange(n_dst) * 7 % n_src).astype(np.int32)
    dQ1, dK1, dV1 = oracle.backward(ip1, ix1, Q, K, V, dO)
    assert np.max(np.abs(dQ1)) < 1e-15 and np.max(np.abs(dK1)) < 1e-15
    ref = np.zeros_like(V)
    np.add.at(ref, ix1, dO)
    np.testing.assert_allclose(dV1, ref, rtol=0, atol=1e-15)
