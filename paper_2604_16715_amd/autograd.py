"""torch.autograd plumbing over the C ABI: the fused attention and the full layer as differentiable
functions.  No arithmetic happens here — forward and backward are the library's entry points; this
module only saves what the backward needs and hands gradients back to autograd."""
from __future__ import annotations

import torch

from .binding import Plan, gta_attn_bwd, gta_attn_fwd, gta_sga_layer_bwd, gta_sga_layer_fwd


class _SparseGraphAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, K, V, plan: Plan, scale: float):
        Q, K, V = Q.contiguous(), K.contiguous(), V.contiguous()
        out, lse = gta_attn_fwd(plan, Q, K, V, scale)
        ctx.save_for_backward(Q, K, V, out, lse)
        ctx.plan, ctx.scale = plan, scale
        ctx.mark_non_differentiable(lse)
        return out, lse

    @staticmethod
    def backward(ctx, d_out, _d_lse):
        Q, K, V, out, lse = ctx.saved_tensors
        dQ, dK, dV = gta_attn_bwd(ctx.plan, Q, K, V, out, lse, d_out.contiguous(), ctx.scale)
        return dQ, dK, dV, None, None


def sparse_graph_attention(plan: Plan, Q, K, V, scale: float = 0.0, return_lse: bool = False):
    """out [n_dst, H, D] = softmax over each row's stored entries of (Q K^T * scale) times V
    (Eq. 4-5), differentiable in Q, K and V.  scale <= 0 selects 1/sqrt(head_dim)."""
    out, lse = _SparseGraphAttention.apply(Q, K, V, plan, scale)
    return (out, lse) if return_lse else out


class _SGALayer(torch.autograd.Function):
    @staticmethod
    def forward(ctx, X, Wq, Wk, Wv, Wo, plan: Plan, heads: int, scale: float):
        X = X.contiguous()
        Ws = [w.contiguous() for w in (Wq, Wk, Wv, Wo)]
        Xout, saved = gta_sga_layer_fwd(plan, X, *Ws, heads, scale)
        ctx.save_for_backward(X, *Ws, saved["Q"], saved["K"], saved["V"], saved["Y"], saved["lse"])
        ctx.plan, ctx.heads, ctx.scale = plan, heads, scale
        return Xout

    @staticmethod
    def backward(ctx, dXout):
        X, Wq, Wk, Wv, Wo, Q, K, V, Y, lse = ctx.saved_tensors
        saved = dict(Q=Q, K=K, V=V, Y=Y, lse=lse)
        dX, dWq, dWk, dWv, dWo = gta_sga_layer_bwd(ctx.plan, X, Wq, Wk, Wv, Wo, saved, dXout.contiguous(),
                                                   ctx.heads, ctx.scale)
        cast = lambda g, w: g.to(w.dtype)   # weight gradients come back in float32
        return dX, cast(dWq, Wq), cast(dWk, Wk), cast(dWv, Wv), cast(dWo, Wo), None, None, None


class SGALayer(torch.nn.Module):
    """One Sparse Graph Attention layer (Eq. 3-5): X' = X W_o + attention(X W_Q, X W_K, X W_V) over the
    plan's graph (n_src == n_dst).  Weights are [d, d] (input x output), d = heads * head_dim."""

    def __init__(self, d: int, heads: int, dtype=torch.bfloat16, device="cuda", scale: float = 0.0):
        super().__init__()
        if d % heads:
            raise ValueError("d must be a multiple of heads")
        self.heads, self.scale = heads, scale
        mk = lambda: torch.nn.Parameter((torch.randn(d, d, device=device) / d ** 0.5).to(dtype))
        self.Wq, self.Wk, self.Wv, self.Wo = mk(), mk(), mk(), mk()

    def forward(self, plan: Plan, X):
        return _SGALayer.apply(X, self.Wq, self.Wk, self.Wv, self.Wo, plan, self.heads, self.scale)
