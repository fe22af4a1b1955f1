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

namespace {
// Layer scratch: [attention scratch | weight-gradient partials] (whichever is larger; never in use at the
// same time), then the repacked weights of the grouped projections (bfloat16 layers with d in {64, 128, 256}).
struct LayerScratch { size_t shared, pack, total; };
LayerScratch layer_scratch(const gta_plan* plan, int heads, int head_dim, gta_dtype dtype) {
    LayerScratch L{0, 0, 0};
    const size_t attn = gta_attn_scratch_bytes(plan, heads, head_dim, dtype);
    if (attn == 0) return L;
    const int d = heads * head_dim;
    const size_t dw = gta_linear_dw_group_scratch_bytes(plan->n_dst, d, d, 4);
    L.shared = ((attn > dw ? attn : dw) + 255) & ~(size_t)255;
    L.pack = proj_group_supported(d, dtype) ? proj_group_scratch_bytes(d, 4) : 0;
    L.total = L.shared + L.pack;
    return L;
}
}  // namespace

extern "C" GTA_API size_t gta_sga_layer_scratch_bytes(const gta_plan* plan, int heads, int head_dim, gta_dtype dtype) {
    if (!plan) return 0;
    return layer_scratch(plan, heads, head_dim, dtype).total;
}

extern "C" GTA_API gta_status gta_sga_layer_fwd(const gta_plan* plan, const int64_t* indptr, const int32_t* indices,
                                                const void* X, const void* Wq, const void* Wk, const void* Wv,
                                                const void* Wo, void* Q, void* K, void* V, void* Y, float* lse,
                                                void* Xout, int64_t n, int heads, int head_dim, gta_dtype dtype,
                                                float scale, void* scratch, size_t scratch_bytes, void* stream) {
    gta_status rc = check_layer(plan, n, heads, head_dim, dtype);
    if (rc != GTA_OK) return rc;
    const int d = heads * head_dim;
    const LayerScratch L = layer_scratch(plan, heads, head_dim, dtype);
    if (L.total == 0) return fail(GTA_ERR_UNSUPPORTED, "unsupported shape for the layer form");
    if (!scratch || scratch_bytes < L.total)
        return fail(GTA_ERR_WORKSPACE, "scratch has %zu bytes, %zu needed", scratch_bytes, L.total);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (L.pack > 0) {
        // Q, K, V from one read of X (Eq. 3)
        void* pack = static_cast<char*>(scratch) + L.shared;
        const void* xs[1] = {X};
        const void* wqkv[3] = {Wq, Wk, Wv};
        void* qkv[3] = {Q, K, V};
        if ((rc = proj_group(xs, 1, wqkv, 3, nullptr, qkv, n, d, 0, pack, L.pack, st)) != GTA_OK) return rc;
        if ((rc = gta_attn_fwd(plan, indptr, indices, Q, K, V, Y, lse, n, n, heads, head_dim, dtype, scale, scratch,
                               L.shared, stream)) != GTA_OK)
            return rc;
        // one product with an addend: the single-projection kernel is the faster of the two forms
        return gta_linear(X, Wo, Y, Xout, n, d, d, dtype, 0, stream);
    }
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
    const LayerScratch L = layer_scratch(plan, heads, head_dim, dtype);
    if (L.total == 0) return fail(GTA_ERR_UNSUPPORTED, "unsupported shape for the layer form");
    if (!scratch || scratch_bytes < L.total)
        return fail(GTA_ERR_WORKSPACE, "scratch has %zu bytes, %zu needed", scratch_bytes, L.total);
    // X' = X W_o + Y:  dY = dX',  dW_o = X^T dX',  dX = dX' W_o^T
    if ((rc = gta_attn_bwd(plan, indptr, indices, Q, K, V, Y, lse, dXout, dQ, dK, dV, n, n, heads, head_dim, dtype,
                           scale, scratch, L.shared, stream)) != GTA_OK)
        return rc;
    {
        // the four weight gradients X^T dX', X^T dQ, X^T dK, X^T dV share X: one launch
        const void* xs[4] = {X, X, X, X};
        const void* dys[4] = {dXout, dQ, dK, dV};
        float* dws[4] = {dWo, dWq, dWk, dWv};
        if ((rc = gta_linear_dw_group(xs, dys, dws, 4, n, d, d, dtype, scratch, L.shared, stream)) != GTA_OK) return rc;
    }
    if (L.pack > 0) {
        // dX = dX' W_o^T + dQ W_Q^T + dK W_K^T + dV W_V^T: one kernel, summed in fp32, rounded once
        const void* ins[4] = {dXout, dQ, dK, dV};
        const void* ws[4] = {Wo, Wq, Wk, Wv};
        void* out[1] = {dX};
        return proj_group(ins, 4, ws, 1, nullptr, out, n, d, 1, static_cast<char*>(scratch) + L.shared, L.pack,
                          static_cast<hipStream_t>(stream));
    }
    // other shapes: accumulated through the addend (in place), rounded to the tensor type after each product
    if ((rc = gta_linear(dXout, Wo, nullptr, dX, n, d, d, dtype, 1, stream)) != GTA_OK) return rc;
    if ((rc = gta_linear(dQ, Wq, dX, dX, n, d, d, dtype, 1, stream)) != GTA_OK) return rc;
    if ((rc = gta_linear(dK, Wk, dX, dX, n, d, d, dtype, 1, stream)) != GTA_OK) return rc;
    return gta_linear(dV, Wv, dX, dX, n, d, d, dtype, 1, stream);
}
