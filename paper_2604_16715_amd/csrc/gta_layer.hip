// One Sparse Graph Attention layer (paper Eq. 3-5) composed from the library's own entry points:
//   Q,K,V = X W_Q, X W_K, X W_V        (three MFMA projections)
//   Y     = attention(Q, K, V; A)      (fused SDDMM -> softmax -> SpMM)
//   X'    = X W_o + Y                  (MFMA projection with the attention output as addend)
// and its backward.  Host-side sequencing only; every step is a kernel of this library.  The
// layer form assumes every source row is an owned row (n_src == n_dst): projecting halo rows is
// the owning GPU's work (Algorithm 1).
#include "gta_internal.h"

using namespace gta;

namespace {
gta_status check_layer(const gta_plan* plan, int64_t n, int heads, int head_dim, gta_dtype dtype) {
    if (!plan) return fail(GTA_ERR_INVALID_ARG, "plan is null");
    if (plan->n_dst != n || plan->n_src != n)
        return fail(GTA_ERR_INVALID_ARG, "the layer form needs n_src == n_dst == n (plan has %lld, %lld)",
                    (long long)plan->n_dst, (long long)plan->n_src);
    if (dtype != GTA_BF16 && dtype != GTA_F32) return fail(GTA_ERR_UNSUPPORTED, "unknown dtype %d", (int)dtype);
    if (heads <= 0 || head_dim <= 0) return fail(GTA_ERR_INVALID_ARG, "heads and head_dim must be positive");
    return GTA_OK;
}
}  // namespace

extern "C" GTA_API size_t gta_sga_layer_scratch_bytes(const gta_plan* plan, int heads, int head_dim, gta_dtype dtype) {
    if (!plan) return 0;
    const size_t attn = gta_attn_scratch_bytes(plan, heads, head_dim, dtype);
    if (attn == 0) return 0;
    const int d = heads * head_dim;
    const size_t dw = gta_linear_dw_scratch_bytes(plan->n_dst, d, d);
    return attn > dw ? attn : dw;
}

extern "C" GTA_API gta_status gta_sga_layer_fwd(const gta_plan* plan, const int64_t* indptr, const int32_t* indices,
                                                const void* X, const void* Wq, const void* Wk, const void* Wv,
                                                const void* Wo, void* Q, void* K, void* V, void* Y, float* lse,
                                                void* Xout, int64_t n, int heads, int head_dim, gta_dtype dtype,
                                                float scale, void* scratch, size_t scratch_bytes, void* stream) {
    gta_status rc = check_layer(plan, n, heads, head_dim, dtype);
    if (rc != GTA_OK) return rc;
    const int d = heads * head_dim;
    if ((rc = gta_linear(X, Wq, nullptr, Q, n, d, d, dtype, 0, stream)) != GTA_OK) return rc;
    if ((rc = gta_linear(X, Wk, nullptr, K, n, d, d, dtype, 0, stream)) != GTA_OK) return rc;
    if ((rc = gta_linear(X, Wv, nullptr, V, n, d, d, dtype, 0, stream)) != GTA_OK) return rc;
    if ((rc = gta_attn_fwd(plan, indptr, indices, Q, K, V, Y, lse, n, n, heads, head_dim, dtype, scale, scratch,
                           scratch_bytes, stream)) != GTA_OK)
        return rc;
    return gta_linear(X, Wo, Y, Xout, n, d, d, dtype, 0, stream);
}

extern "C" GTA_API gta_status gta_sga_layer_bwd(const gta_plan* plan, const int64_t* indptr, const int32_t* indices,
                                                const void* X, const void* Wq, const void* Wk, const void* Wv,
                                                const void* Wo, const void* Q, const void* K, const void* V,
                                                const void* Y, const float* lse, const void* dXout, void* dQ,
                                                void* dK, void* dV, void* dX, float* dWq, float* dWk, float* dWv,
                                                float* dWo, int64_t n, int heads, int head_dim, gta_dtype dtype,
                                                float scale, void* scratch, size_t scratch_bytes, void* stream) {
    gta_status rc = check_layer(plan, n, heads, head_dim, dtype);
    if (rc != GTA_OK) return rc;
    const int d = heads * head_dim;
    if (scratch_bytes < gta_sga_layer_scratch_bytes(plan, heads, head_dim, dtype) &&
        scratch_bytes < gta_linear_dw_scratch_bytes(n, d, d))
        return fail(GTA_ERR_WORKSPACE, "scratch too small for the weight gradients");
    // X' = X W_o + Y:  dY = dX',  dW_o = X^T dX',  dX = dX' W_o^T
    if ((rc = gta_attn_bwd(plan, indptr, indices, Q, K, V, Y, lse, dXout, dQ, dK, dV, n, n, heads, head_dim, dtype,
                           scale, scratch, scratch_bytes, stream)) != GTA_OK)
        return rc;
    if ((rc = gta_linear_dw(X, dXout, dWo, n, d, d, dtype, scratch, scratch_bytes, stream)) != GTA_OK) return rc;
    if ((rc = gta_linear_dw(X, dQ, dWq, n, d, d, dtype, scratch, scratch_bytes, stream)) != GTA_OK) return rc;
    if ((rc = gta_linear_dw(X, dK, dWk, n, d, d, dtype, scratch, scratch_bytes, stream)) != GTA_OK) return rc;
    if ((rc = gta_linear_dw(X, dV, dWv, n, d, d, dtype, scratch, scratch_bytes, stream)) != GTA_OK) return rc;
    // dX = dX' W_o^T + dQ W_Q^T + dK W_K^T + dV W_V^T, accumulated through the addend (in place)
    if ((rc = gta_linear(dXout, Wo, nullptr, dX, n, d, d, dtype, 1, stream)) != GTA_OK) return rc;
    if ((rc = gta_linear(dQ, Wq, dX, dX, n, d, d, dtype, 1, stream)) != GTA_OK) return rc;
    if ((rc = gta_linear(dK, Wk, dX, dX, n, d, d, dtype, 1, stream)) != GTA_OK) return rc;
    return gta_linear(dV, Wv, dX, dX, n, d, d, dtype, 1, stream);
}
