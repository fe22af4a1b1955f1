"""The Python binding refuses mismatched tensors before anything reaches the C ABI (which takes raw
pointers and could not see the mismatch).  Runs without a GPU: a stand-in plan object and CPU
tensors are enough, because every check fires before the first library call."""
import pytest
import torch

import paper_2604_16715_amd as gta
from paper_2604_16715_amd import binding


class FakePlan:
    """Carries what the checks read from a Plan; handle is None so a call that got past the checks
    would fail in ctypes rather than run."""

    def __init__(self, n_dst, n_src, nnz):
        self.n_dst, self.n_src = n_dst, n_src
        self.indptr = torch.zeros(n_dst + 1, dtype=torch.int64)
        self.indices = torch.zeros(nnz, dtype=torch.int32)
        self.handle = None

    def scratch(self, *a, **k):   # pragma: no cover - reaching this means a check was missed
        raise AssertionError("a mismatched call got past the argument checks")


def t(*shape, dtype=torch.float32):
    return torch.zeros(shape, dtype=dtype)


def test_forward_mismatches_raise_before_launch():
    plan = FakePlan(6, 9, 20)
    Q, K, V = t(6, 4, 16), t(9, 4, 16), t(9, 4, 16)
    bad = [
        dict(Q=t(5, 4, 16)),                                   # rows differ from the plan
        dict(K=t(8, 4, 16)),                                   # source rows differ
        dict(K=t(9, 2, 16)),                                   # other head count
        dict(V=t(9, 4, 8)),                                    # other head_dim
        dict(K=t(9, 4, 16, dtype=torch.bfloat16)),             # dtype differs from Q's
        dict(V=t(9, 4, 32)[:, :, ::2]),                        # non-contiguous view
        dict(K=t(9, 8, 16)[:, ::2]),
        dict(Q=t(6, 64)),                                      # not [rows, heads, head_dim]
    ]
    for change in bad:
        args = dict(Q=Q, K=K, V=V)
        args.update(change)
        with pytest.raises(gta.GtaError):
            gta.gta_attn_fwd(plan, args["Q"], args["K"], args["V"])
    with pytest.raises(gta.GtaError):
        gta.gta_attn_fwd(plan, Q, K, V, out=t(6, 4, 16), lse=t(6, 4, dtype=torch.float64))
    with pytest.raises(gta.GtaError):
        gta.gta_attn_fwd(plan, Q, K, V, out=t(6, 4, 8))
    with pytest.raises(gta.GtaError):
        gta.gta_attn_fwd_noalloc(plan, Q, K, V, t(6, 4, 16), t(6, 3))
    with pytest.raises(gta.GtaError):
        gta.gta_attn_fwd(plan, Q.to(torch.float16), K.to(torch.float16), V.to(torch.float16))


def test_backward_and_halo_mismatches_raise():
    plan = FakePlan(6, 9, 20)
    Q, K, V, out, lse, dO = t(6, 4, 16), t(9, 4, 16), t(9, 4, 16), t(6, 4, 16), t(6, 4), t(6, 4, 16)
    with pytest.raises(gta.GtaError):
        gta.gta_attn_bwd(plan, Q, K, V, out, lse, t(6, 4, 8))
    with pytest.raises(gta.GtaError):
        gta.gta_attn_bwd(plan, Q, K, V, out, t(6, 2), dO)
    with pytest.raises(gta.GtaError):
        gta.gta_attn_bwd(plan, Q, K, V, out, lse, dO, dK=t(6, 4, 16))
    with pytest.raises(gta.GtaError):
        gta.gta_attn_bwd(plan, Q, K, V, out.to(torch.bfloat16), lse, dO)
    # halo forms: the two parts must add up to the plan's source rows and agree in shape
    with pytest.raises(gta.GtaError):
        gta.gta_attn_fwd_halo(plan, Q, t(6, 4, 16), t(6, 4, 16), t(2, 4, 16), t(2, 4, 16))
    with pytest.raises(gta.GtaError):
        gta.gta_attn_fwd_halo(plan, Q, t(6, 4, 16), t(6, 4, 16), t(3, 4, 16), t(3, 2, 16))
    with pytest.raises(gta.GtaError):
        gta.gta_attn_bwd_halo(plan, Q, t(6, 4, 16), t(6, 4, 16), t(3, 4, 16), t(3, 4, 16), out, lse, t(5, 4, 16))


def test_operator_and_projection_mismatches_raise():
    plan = FakePlan(6, 9, 20)
    with pytest.raises(gta.GtaError):
        gta.gta_sddmm(plan, t(6, 4, 16), t(9, 4, 8))
    with pytest.raises(gta.GtaError):
        gta.gta_edge_softmax(plan, t(19, 4), 1.0)              # not nnz rows
    with pytest.raises(gta.GtaError):
        gta.gta_edge_softmax_bwd(plan, t(20, 4), t(20, 2), 1.0)
    with pytest.raises(gta.GtaError):
        gta.gta_spmm(plan, t(20, 2), t(9, 4, 16))              # weights for another head count
    with pytest.raises(gta.GtaError):
        gta.gta_spmm(plan, t(20, 4), t(9, 4, 16), transposed=True)   # transposed reads [n_dst, ...]
    with pytest.raises(gta.GtaError):
        gta.gta_linear(t(10, 32), t(16, 32))                   # W is [d_in, d_out] unless trans_w
    with pytest.raises(gta.GtaError):
        gta.gta_linear(t(10, 32), t(32, 16, dtype=torch.bfloat16))   # weight dtype differs from X's
    with pytest.raises(gta.GtaError):
        gta.gta_linear(t(10, 32), t(32, 16), C=t(10, 8))
    with pytest.raises(gta.GtaError):
        gta.gta_linear_dw(t(10, 32), t(9, 16))
    sq = FakePlan(6, 6, 20)
    W = t(64, 64)
    with pytest.raises(gta.GtaError):                          # fp32 X with bf16 weights
        gta.gta_sga_layer_fwd(sq, t(6, 64), W.to(torch.bfloat16), W, W, W, heads=4)
    with pytest.raises(gta.GtaError):
        gta.gta_sga_layer_fwd(sq, t(6, 64), W, W, t(64, 32), W, heads=4)
    with pytest.raises(gta.GtaError):
        gta.gta_sga_layer_fwd(plan, t(6, 64), W, W, W, W, heads=4)   # needs n_src == n_dst
    with pytest.raises(gta.GtaError):
        gta.gta_attn_merge(t(6, 4, 16), t(6, 4), t(6, 4, 16), t(6, 2))
    with pytest.raises(gta.GtaError):
        gta.gta_head_split(t(6, 4, 16), 2, S=t(2, 6, 4, 16))


def test_plan_create_checks_and_validates_by_default():
    import inspect
    assert inspect.signature(gta.gta_plan_create).parameters["validate"].default is True
    with pytest.raises(gta.GtaError):
        gta.gta_plan_create(torch.zeros(4, dtype=torch.int32), torch.zeros(3, dtype=torch.int32), 3)
    with pytest.raises(gta.GtaError):   # CPU tensors are refused before the library sees them
        gta.gta_plan_create(torch.zeros(4, dtype=torch.int64), torch.zeros(3, dtype=torch.int32), 3)
    assert binding._need is not None
