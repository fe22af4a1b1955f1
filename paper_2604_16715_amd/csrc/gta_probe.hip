// Streaming probes: the bandwidth a plain kernel reaches on this GPU, measured beside the attention
// passes so that their throughput can be read against an achievable ceiling as well as against the
// published HBM peak.  Three access mixes: read only (the attention passes are read-dominated),
// copy (one read, one write) and add (two reads, one write).  16 bytes per lane, four independent
// accesses per thread, non-temporal (every byte is touched once).
#include "gta_internal.h"

namespace gta {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int kProbeThreads = 256, kProbeUnroll = 4;

// MODE 0: read a, fold into one value per thread (stored only if it is a chosen bit pattern, so the
//         loads cannot be dropped and nothing is written in practice);  1: dst = a;  2: dst = a + b
template <int MODE>
__global__ void __launch_bounds__(kProbeThreads)
k_probe(u32x4* __restrict__ dst, const u32x4* __restrict__ a, const u32x4* __restrict__ b, int64_t n_units) {
    const int64_t base = (int64_t)blockIdx.x * (kProbeThreads * kProbeUnroll) + threadIdx.x;
    u32x4 x[kProbeUnroll], y[kProbeUnroll];
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) {
        const int64_t i = base + (int64_t)u * kProbeThreads;
        x[u] = u32x4{0, 0, 0, 0};
        y[u] = u32x4{0, 0, 0, 0};
        if (i < n_units) {
            x[u] = __builtin_nontemporal_load(a + i);
            if (MODE == 2) y[u] = __builtin_nontemporal_load(b + i);
        }
    }
    if (MODE == 0) {
        unsigned int fold = 0;
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) fold ^= x[u].x ^ x[u].y ^ x[u].z ^ x[u].w;
        if (fold == 0x9E3779B9u && base < n_units) dst[0] = u32x4{fold, fold, fold, fold};
        return;
    }
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) {
        const int64_t i = base + (int64_t)u * kProbeThreads;
        if (i >= n_units) continue;
        u32x4 r = x[u];
        if (MODE == 2) {
            r.x = __float_as_uint(__uint_as_float(x[u].x) + __uint_as_float(y[u].x));
            r.y = __float_as_uint(__uint_as_float(x[u].y) + __uint_as_float(y[u].y));
            r.z = __float_as_uint(__uint_as_float(x[u].z) + __uint_as_float(y[u].z));
            r.w = __float_as_uint(__uint_as_float(x[u].w) + __uint_as_float(y[u].w));
        }
        __builtin_nontemporal_store(r, dst + i);
    }
}

}  // namespace
}  // namespace gta

using namespace gta;

extern "C" GTA_API gta_status gta_stream_probe(int mode, void* dst, const void* a, const void* b, size_t bytes,
                                               void* stream) {
    if (mode < 0 || mode > 2) return fail(GTA_ERR_INVALID_ARG, "mode must be 0 (read), 1 (copy) or 2 (add)");
    if (!dst || !a || (mode == 2 && !b)) return fail(GTA_ERR_INVALID_ARG, "null pointer argument");
    if (((uintptr_t)dst & 15) || ((uintptr_t)a & 15) || ((uintptr_t)b & 15) || (bytes & 15))
        return fail(GTA_ERR_INVALID_ARG, "pointers and size must be multiples of 16 bytes");
    const int64_t n_units = (int64_t)(bytes / 16);
    if (n_units == 0) return GTA_OK;
    const int64_t per_block = kProbeThreads * kProbeUnroll;
    const int64_t blocks = (n_units + per_block - 1) / per_block;
    if (blocks > 0x7FFFFFFFll) return fail(GTA_ERR_UNSUPPORTED, "probe size too large");
    hipStream_t st = static_cast<hipStream_t>(stream);
    LaunchTimer t(mode == 0 ? "probe_read" : mode == 1 ? "probe_copy" : "probe_add", 0, n_units, st);
    const dim3 grid((unsigned)blocks), block(kProbeThreads);
    if (mode == 0)
        hipLaunchKernelGGL(k_probe<0>, grid, block, 0, st, (u32x4*)dst, (const u32x4*)a, (const u32x4*)b, n_units);
    else if (mode == 1)
        hipLaunchKernelGGL(k_probe<1>, grid, block, 0, st, (u32x4*)dst, (const u32x4*)a, (const u32x4*)b, n_units);
    else
        hipLaunchKernelGGL(k_probe<2>, grid, block, 0, st, (u32x4*)dst, (const u32x4*)a, (const u32x4*)b, n_units);
    GTA_HIP_TRY(hipGetLastError());
    return GTA_OK;
}
