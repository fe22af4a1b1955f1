// Layout transforms of GP-A2A (paper Section 3.2, Algorithm 2): the all-to-all turns a node-split
// tensor [(N/p), h, d'] into a head-split one [N, (h/p), d'].  On the sending side that means
// regrouping each local row's heads into p contiguous blocks (one per destination GPU); on the
// receiving side the blocks of the p senders concatenate by rows, which needs no kernel.  The
// reverse transform restores [(N/p), h, d'] from p received head blocks.  Pure data movement,
// 16 bytes per lane, bound by HBM bandwidth.
#include "gta_internal.h"

namespace gta {
namespace {

// split: S[part][row][c] = X[row][part * per + c]   merge: the inverse.  Units of 16 bytes.
template <bool SPLIT>
__global__ void __launch_bounds__(256)
k_head_regroup(const uint4* __restrict__ in, uint4* __restrict__ out, int64_t n_rows, int units_per_row,
               int units_per_part) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_rows * units_per_row) return;
    const int64_t row = i / units_per_row;
    const int c = (int)(i - row * units_per_row);
    const int part = c / units_per_part, within = c - part * units_per_part;
    const int64_t split_index = ((int64_t)part * n_rows + row) * units_per_part + within;
    if (SPLIT) out[split_index] = in[i];
    else out[i] = in[split_index];
}

gta_status regroup(bool split, const void* in, void* out, int64_t n_rows, int heads, int head_dim,
                   gta_dtype dtype, int parts, void* stream) {
    if (dtype != GTA_F32 && dtype != GTA_BF16) return fail(GTA_ERR_UNSUPPORTED, "unknown dtype %d", (int)dtype);
    if (n_rows < 0 || heads <= 0 || head_dim <= 0 || parts <= 0) return fail(GTA_ERR_INVALID_ARG, "bad sizes");
    if (heads % parts != 0) return fail(GTA_ERR_INVALID_ARG, "heads (%d) must be divisible by parts (%d)", heads, parts);
    const int64_t part_bytes = (int64_t)(heads / parts) * head_dim * (dtype == GTA_F32 ? 4 : 2);
    if (part_bytes % 16 != 0) return fail(GTA_ERR_UNSUPPORTED, "a head block must be a multiple of 16 bytes");
    if (n_rows == 0) return GTA_OK;
    if (!in || !out) return fail(GTA_ERR_INVALID_ARG, "null tensor pointer");
    if (((uintptr_t)in & 15) || ((uintptr_t)out & 15)) return fail(GTA_ERR_INVALID_ARG, "tensor base pointers must be 16-byte aligned");
    const int units_per_part = (int)(part_bytes / 16), units_per_row = units_per_part * parts;
    const int64_t total = n_rows * units_per_row;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    hipStream_t st = static_cast<hipStream_t>(stream);
    LaunchTimer t(split ? "head_split" : "head_merge", n_rows, 0, st);
    if (split)
        hipLaunchKernelGGL(k_head_regroup<true>, dim3(blocks), dim3(256), 0, st, (const uint4*)in, (uint4*)out,
                           n_rows, units_per_row, units_per_part);
    else
        hipLaunchKernelGGL(k_head_regroup<false>, dim3(blocks), dim3(256), 0, st, (const uint4*)in, (uint4*)out,
                           n_rows, units_per_row, units_per_part);
    GTA_HIP_TRY(hipGetLastError());
    return GTA_OK;
}

}  // namespace
}  // namespace gta

extern "C" GTA_API gta_status gta_head_split(const void* X, void* S, int64_t n_rows, int heads, int head_dim,
                                             gta_dtype dtype, int parts, void* stream) {
    return gta::regroup(true, X, S, n_rows, heads, head_dim, dtype, parts, stream);
}

extern "C" GTA_API gta_status gta_head_merge(const void* S, void* X, int64_t n_rows, int heads, int head_dim,
                                             gta_dtype dtype, int parts, void* stream) {
    return gta::regroup(false, S, X, n_rows, heads, head_dim, dtype, parts, stream);
}
