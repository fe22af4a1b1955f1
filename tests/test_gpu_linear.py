"""MFMA projections (X W, X W^T, X^T dY) against the float64 reference."""
import numpy as np
import pytest
import torch

import gen
from helpers import assert_close, to_f64, to_torch
from oracle import dense_ref

pytestmark = pytest.mark.gpu


def bf16_matrix(rows, cols, seed, stream, scale=1.0):
    x = gen.normal((rows, cols), "bf16", seed, stream)
    if scale != 1.0:
        f = (gen.bf16_bits_to_f32(x) * scale).astype(np.float32)
        x = (f.view(np.uint32) >> 16).astype(np.uint16)   # truncation keeps the values exactly representable
    return x


@pytest.mark.parametrize("n,d_in,d_out", [
    (1000, 128, 128), (4097, 256, 256), (333, 64, 64), (2048, 256, 768), (513, 128, 384), (129, 512, 512),
    (64, 16, 8), (1, 32, 40), (5000, 48, 200),
    # enough rows that a wavefront walks over several tiles (run-ahead loop, odd and even tile counts, ragged end)
    (150001, 128, 128), (200003, 256, 256), (140000, 256, 64), (131073, 64, 128), (197000, 128, 64),
])
def test_linear_forward_forms(n, d_in, d_out):
    import paper_2604_16715_amd as gta
    print(f"linear case n={n} d_in={d_in} d_out={d_out}", flush=True)
    X, W, C = bf16_matrix(n, d_in, 1, 2), bf16_matrix(d_in, d_out, 1, 3, 0.125), bf16_matrix(n, d_out, 1, 4)
    Xf, Wf, Cf = (gen.bf16_bits_to_f32(a).astype(np.float64) for a in (X, W, C))
    Xd, Wd, Cd = to_torch(X), to_torch(W), to_torch(C)
    assert_close("X W", to_f64(gta.gta_linear(Xd, Wd)), dense_ref.linear(Xf, Wf), 2e-2)
    assert_close("X W + C", to_f64(gta.gta_linear(Xd, Wd, Cd)), dense_ref.linear(Xf, Wf, Cf), 2e-2)
    Wt = to_torch(np.ascontiguousarray(W.T))
    assert_close("X W^T form", to_f64(gta.gta_linear(Xd, Wt, Cd, trans_w=True)), dense_ref.linear(Xf, Wf, Cf), 2e-2)
    # results of the two storage forms of W are the same bits: same products, same order
    assert torch.equal(gta.gta_linear(Xd, Wd, Cd).view(torch.int16), gta.gta_linear(Xd, Wt, Cd, trans_w=True).view(torch.int16))


@pytest.mark.parametrize("n,d_in,d_out", [
    (1000, 128, 128), (70000, 256, 256), (333, 64, 192), (31, 16, 8), (4096, 512, 128), (5000, 48, 200),
    (97, 256, 256), (129, 144, 256), (200000, 256, 176), (7, 256, 8),
])
def test_linear_weight_gradient(n, d_in, d_out):
    import paper_2604_16715_amd as gta
    print(f"linear_dw case n={n} d_in={d_in} d_out={d_out}", flush=True)
    X, dY = bf16_matrix(n, d_in, 2, 2), bf16_matrix(n, d_out, 2, 5)
    Xf, dYf = (gen.bf16_bits_to_f32(a).astype(np.float64) for a in (X, dY))
    got = gta.gta_linear_dw(to_torch(X), to_torch(dY))
    assert_close("X^T dY", to_f64(got), dense_ref.linear_dw(Xf, dYf), 1e-4)
    again = gta.gta_linear_dw(to_torch(X), to_torch(dY))
    assert torch.equal(got, again), "weight gradient is not bitwise reproducible"


def test_linear_rejects_unsupported():
    import paper_2604_16715_amd as gta
    X = torch.zeros((8, 24), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((24, 16), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(gta.GtaError):
        gta.gta_linear(X, W)                     # d_in not a multiple of 16
    X = torch.zeros((8, 512), dtype=torch.float32, device="cuda")
    W = torch.zeros((512, 16), dtype=torch.float32, device="cuda")
    with pytest.raises(gta.GtaError):
        gta.gta_linear(X, W)                     # fp32 weight panel of 64 x 512 does not fit in LDS


@pytest.mark.parametrize("n,d", [(257, 256), (1025, 256), (70001, 256), (129, 128), (66000 + 33, 128), (130, 64), (5, 48)])
def test_linear_accumulates_in_place(n, d):
    """Y may alias C (dX += dY W^T in the layer's backward).  n is chosen so that whole wavefronts of the
    last row block lie past the end: they must not touch the last row."""
    import paper_2604_16715_amd as gta
    print(f"linear in-place case n={n} d={d}", flush=True)
    X, W, C = bf16_matrix(n, d, 3, 2), bf16_matrix(d, d, 3, 3, 0.125), bf16_matrix(n, d, 3, 4)
    Xd, Wd = to_torch(X), to_torch(W)
    for trans in (False, True):
        ref = gta.gta_linear(Xd, Wd, to_torch(C), trans_w=trans)
        for _ in range(3):
            acc = to_torch(C)
            out = gta.gta_linear(Xd, Wd, acc, trans_w=trans, Y=acc)
            torch.cuda.synchronize()
            assert out.data_ptr() == acc.data_ptr()
            assert torch.equal(out.view(torch.int16), ref.view(torch.int16))



# ---- fp32 forms (v_mfma_f32_32x32x2_f32).  Tolerance: fp32 accumulation over d_in <= 496 terms per
# output (and, for X^T dY, row splits of a few hundred rows summed in a second step) keeps the normwise
# error near sqrt(terms) * 2^-24, i.e. ~1e-6; gated at the attention path's fp32 bar.
F32_TOL = 1e-5


def f32_matrix(rows, cols, seed, stream, scale=1.0):
    return (gen.normal((rows, cols), "f32", seed, stream) * np.float32(scale)).astype(np.float32)


@pytest.mark.parametrize("n,d_in,d_out", [
    (1000, 128, 128), (4097, 256, 256), (333, 64, 64), (2048, 64, 192), (129, 496, 72), (64, 16, 8), (1, 32, 40),
    (5000, 48, 200), (169343, 128, 128), (140001, 64, 64),
])
def test_linear_forward_forms_f32(n, d_in, d_out):
    import paper_2604_16715_amd as gta
    print(f"linear f32 case n={n} d_in={d_in} d_out={d_out}", flush=True)
    X, W, C = f32_matrix(n, d_in, 7, 2), f32_matrix(d_in, d_out, 7, 3, 0.125), f32_matrix(n, d_out, 7, 4)
    Xf, Wf, Cf = (a.astype(np.float64) for a in (X, W, C))
    Xd, Wd, Cd = to_torch(X), to_torch(W), to_torch(C)
    assert_close("X W", to_f64(gta.gta_linear(Xd, Wd)), dense_ref.linear(Xf, Wf), F32_TOL)
    assert_close("X W + C", to_f64(gta.gta_linear(Xd, Wd, Cd)), dense_ref.linear(Xf, Wf, Cf), F32_TOL)
    Wt = to_torch(np.ascontiguousarray(W.T))
    got_t = gta.gta_linear(Xd, Wt, Cd, trans_w=True)
    assert_close("X W^T form", to_f64(got_t), dense_ref.linear(Xf, Wf, Cf), F32_TOL)
    assert torch.equal(gta.gta_linear(Xd, Wd, Cd), got_t)     # same products in the same order
    acc = Cd.clone()                                          # in place
    assert torch.equal(gta.gta_linear(Xd, Wd, acc, Y=acc), got_t)


@pytest.mark.parametrize("n,d_in,d_out", [(1000, 128, 128), (70000, 256, 256), (333, 64, 192), (31, 16, 8), (5000, 48, 200)])
def test_linear_weight_gradient_f32(n, d_in, d_out):
    import paper_2604_16715_amd as gta
    print(f"linear_dw f32 case n={n} d_in={d_in} d_out={d_out}", flush=True)
    X, dY = f32_matrix(n, d_in, 8, 2), f32_matrix(n, d_out, 8, 5)
    got = gta.gta_linear_dw(to_torch(X), to_torch(dY))
    assert_close("X^T dY", to_f64(got), dense_ref.linear_dw(X.astype(np.float64), dY.astype(np.float64)), F32_TOL)
    assert torch.equal(got, gta.gta_linear_dw(to_torch(X), to_torch(dY)))   # fixed summation order


@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("n", [1, 127, 129, 1000, 40001, 150001])
def test_linear_group(n, d):
    """Grouped projections (one launch, every input read once): Q, K, V from one X; a projection with
    addend; the four-term input gradient accumulated in fp32 and rounded once."""
    import paper_2604_16715_amd as gta
    print(f"linear_group case n={n} d={d}", flush=True)
    Xs = [bf16_matrix(n, d, 7, 20 + i) for i in range(4)]
    Ws = [bf16_matrix(d, d, 7, 30 + i, 0.125) for i in range(4)]
    C = bf16_matrix(n, d, 7, 40)
    f = lambda a: gen.bf16_bits_to_f32(a).astype(np.float64)
    Xd, Wd, Cd = [to_torch(a) for a in Xs], [to_torch(a) for a in Ws], to_torch(C)
    # 1 -> 3 (Eq. 3)
    Q, K, V = gta.gta_linear_group([Xd[0]], Wd[:3])
    for name, got, W in zip("QKV", (Q, K, V), Ws[:3]):
        assert_close(name, to_f64(got), dense_ref.linear(f(Xs[0]), f(W)), 2e-2)
    # ... bitwise the single projection's result (same products, same order, one rounding)
    assert torch.equal(K.view(torch.int16), gta.gta_linear(Xd[0], Wd[1]).view(torch.int16))
    # 1 -> 1 with and without addend (Eq. 5), both weight storage orders
    (Y,) = gta.gta_linear_group([Xd[1]], [Wd[3]], [Cd])
    assert_close("X W + C", to_f64(Y), dense_ref.linear(f(Xs[1]), f(Ws[3]), f(C)), 2e-2)
    (Yt,) = gta.gta_linear_group([Xd[1]], [to_torch(np.ascontiguousarray(Ws[3].T))], [Cd], trans_w=True)
    assert torch.equal(Y.view(torch.int16), Yt.view(torch.int16))
    (Y0,) = gta.gta_linear_group([Xd[2]], [Wd[0]])
    assert_close("X W", to_f64(Y0), dense_ref.linear(f(Xs[2]), f(Ws[0])), 2e-2)
    # 4 -> 1: dX = sum_p X_p W_p^T, against the float64 sum (error of ONE bf16 rounding: well inside 2e-2)
    (dX,) = gta.gta_linear_group(Xd, Wd, trans_w=True)
    ref = sum(dense_ref.linear(f(x), f(w), trans_w=True) for x, w in zip(Xs, Ws))
    emax, _ = assert_close("dX", to_f64(dX), ref, 2e-2)
    assert emax < 4e-3   # a single rounding to bf16 (2^-9 relative) of values up to max|ref|
    torch.cuda.synchronize()


@pytest.mark.parametrize("n,d_in,d_out,p", [(40001, 256, 256, 4), (1000, 128, 128, 3), (333, 64, 192, 2), (70000, 256, 128, 4),
                                            (31, 16, 8, 4), (0, 64, 64, 2), (100, 256, 256, 3), (33, 208, 256, 2), (1, 256, 256, 1),
                                            (300001, 256, 256, 2), (0, 256, 256, 2)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_linear_weight_gradient_group(n, d_in, d_out, p, dtype):
    """Several weight gradients in one call (the four of Eq. 3 and 5 share the layer input): each equals,
    bit for bit, the single-product entry point's result, which the tests above hold to the oracle."""
    import paper_2604_16715_amd as gta
    print(f"linear_dw_group case n={n} d_in={d_in} d_out={d_out} p={p} {dtype}", flush=True)
    make = bf16_matrix if dtype == "bf16" else f32_matrix
    f = (lambda a: gen.bf16_bits_to_f32(a).astype(np.float64)) if dtype == "bf16" else (lambda a: a.astype(np.float64))
    X, X2 = make(n, d_in, 8, 2), make(n, d_in, 8, 3)
    dYs = [make(n, d_out, 8, 10 + k) for k in range(p)]
    Xd, X2d, dYd = to_torch(X), to_torch(X2), [to_torch(a) for a in dYs]
    shared = gta.gta_linear_dw_group([Xd] * p, dYd)                       # every product reads the same X
    mixed = gta.gta_linear_dw_group([Xd] * (p - 1) + [X2d], dYd)          # the last one its own
    for k in range(p):
        one = gta.gta_linear_dw(Xd, dYd[k])
        assert torch.equal(shared[k], one), f"product {k}"
        if n:
            assert_close(f"X^T dY[{k}]", to_f64(one), dense_ref.linear_dw(f(X), f(dYs[k])), 1e-4 if dtype == "bf16" else F32_TOL)
        else:
            assert not one.any()
    for k in range(p - 1):
        assert torch.equal(mixed[k], shared[k])
    assert torch.equal(mixed[p - 1], gta.gta_linear_dw(X2d, dYd[p - 1]))
    torch.cuda.synchronize()


def test_linear_weight_gradient_group_rejects():
    import paper_2604_16715_amd as gta
    X = torch.zeros((8, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(gta.GtaError):
        gta.gta_linear_dw_group([X] * 5, [X] * 5)          # at most four products
    dW = torch.zeros((64, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(gta.GtaError):
        gta.gta_linear_dw_group([X, X], [X, X], [dW, dW])  # results must be distinct
    with pytest.raises(gta.GtaError):
        gta.gta_linear_dw_group([X, X], [X])               # one dY per X


def test_linear_group_rejects_unsupported():
    import paper_2604_16715_amd as gta
    X = torch.zeros((8, 96), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((96, 96), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(gta.GtaError):
        gta.gta_linear_group([X], [W])                     # d = 96
    X = torch.zeros((8, 64), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(gta.GtaError):
        gta.gta_linear_group([X, X], [W, W])               # 2 -> 1 is not an instantiated grouping
    with pytest.raises(gta.GtaError):
        gta.gta_linear_group([X], [W], Ys=[X])             # output aliases the input
    Xf = torch.zeros((8, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(gta.GtaError):
        gta.gta_linear_group([Xf], [W.float()])            # bfloat16 only
