// Combining two partial attention results over disjoint sets of stored entries of the same rows
// (Eq. 2 with the sum over N(i) cut in two): the softmax denominators add, so
//     lse = log(exp(lse_a) + exp(lse_b)),   out = exp(lse_a - lse) out_a + exp(lse_b - lse) out_b.
// This is what lets the entries whose sources are already resident (owned rows, Algorithm 1) be
// processed while the halo rows are still in flight: run the forward on each entry set with its own
// plan, then merge.  Streaming kernel, 16 bytes per lane, bound by HBM bandwidth.
#include "gta_kernels.h"

namespace gta {
namespace {

template <class T>
__global__ void __launch_bounds__(256)
k_attn_merge(const uint4* __restrict__ out_a, const float* __restrict__ lse_a, const uint4* __restrict__ out_b,
             const float* __restrict__ lse_b, uint4* out, float* __restrict__ lse, int64_t n_rows,
             int units_per_row, int head_bytes, int heads) {
    constexpr int NV = Elt<T>::NV, EL = 16 / NV;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_rows * units_per_row) return;
    const int64_t row = i / units_per_row;
    const int byte0 = (int)(i - row * units_per_row) * 16;
    float a[NV], b[NV], o[NV];
    Elt<T>::unpack(out_a[i], a);
    Elt<T>::unpack(out_b[i], b);
    int head = -1;
    float wa = 0.f, wb = 0.f;
#pragma unroll
    for (int e = 0; e < NV; ++e) {
        const int byte = byte0 + e * EL, h = byte / head_bytes;
        if (h != head) {   // weights of the head this element belongs to
            head = h;
            const float la = lse_a[row * heads + h], lb = lse_b[row * heads + h];
            const float m = fmaxf(la, lb);
            float l = -INFINITY;
            wa = 0.f;
            wb = 0.f;
            if (m > -INFINITY) {
                const float ea = expf(la - m), eb = expf(lb - m), s = ea + eb;
                wa = ea / s;
                wb = eb / s;
                l = m + logf(s);
            }
            if (byte == h * head_bytes) lse[row * heads + h] = l;   // the lane holding the head's first element
        }
        o[e] = wa * a[e] + wb * b[e];
    }
    out[i] = Elt<T>::pack(o);
}

}  // namespace
}  // namespace gta

using namespace gta;

extern "C" GTA_API gta_status gta_attn_merge(const void* out_a, const float* lse_a, const void* out_b,
                                             const float* lse_b, void* out, float* lse, int64_t n_rows,
                                             int heads, int head_dim, gta_dtype dtype, void* stream) {
    if (dtype != GTA_F32 && dtype != GTA_BF16) return fail(GTA_ERR_UNSUPPORTED, "unknown dtype %d", (int)dtype);
    if (n_rows < 0 || heads <= 0 || head_dim <= 0) return fail(GTA_ERR_INVALID_ARG, "bad sizes");
    const int el = dtype == GTA_F32 ? 4 : 2;
    const int64_t row_bytes = (int64_t)heads * head_dim * el;
    if (row_bytes % 16 != 0) return fail(GTA_ERR_INVALID_ARG, "heads * head_dim * element size must be a multiple of 16 bytes");
    if (row_bytes > (1 << 20)) return fail(GTA_ERR_UNSUPPORTED, "rows up to 1 MiB are supported");
    if (n_rows == 0) return GTA_OK;
    if (!out_a || !lse_a || !out_b || !lse_b || !out || !lse) return fail(GTA_ERR_INVALID_ARG, "null tensor pointer");
    if (((uintptr_t)out_a & 15) || ((uintptr_t)out_b & 15) || ((uintptr_t)out & 15))
        return fail(GTA_ERR_INVALID_ARG, "tensor base pointers must be 16-byte aligned");
    if (lse == lse_a || lse == lse_b) return fail(GTA_ERR_INVALID_ARG, "lse must not alias lse_a or lse_b");
    const int units_per_row = (int)(row_bytes / 16);
    const int64_t total = n_rows * units_per_row;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    hipStream_t st = static_cast<hipStream_t>(stream);
    LaunchTimer t("attn_merge", n_rows, 0, st);
    if (dtype == GTA_F32)
        hipLaunchKernelGGL(k_attn_merge<float>, dim3(blocks), dim3(256), 0, st, (const uint4*)out_a, lse_a,
                           (const uint4*)out_b, lse_b, (uint4*)out, lse, n_rows, units_per_row, head_dim * el, heads);
    else
        hipLaunchKernelGGL(k_attn_merge<bf16_tag>, dim3(blocks), dim3(256), 0, st, (const uint4*)out_a, lse_a,
                           (const uint4*)out_b, lse_b, (uint4*)out, lse, n_rows, units_per_row, head_dim * el, heads);
    GTA_HIP_TRY(hipGetLastError());
    return GTA_OK;
}
