// The dense projections of the layer for fp32 tensors (paper Eq. 3 and Eq. 5; the paper's own
// runs are presumably fp32): v_mfma_f32_32x32x2_f32, fp32 operands and accumulation.  Same
// structure as the bf16 kernels — the weight panel of a column tile lives in LDS, a wavefront
// walks 32-row tiles of X staged through its own LDS patch, the accumulator holds Y transposed
// so a lane owns 16-byte pieces of one row — without their run-ahead machinery: the fp32 matrix
// rate (157 TFLOP/s) bounds these kernels at d = 256, not HBM, and the fp32 workloads are the
// small ones.
//
// Fragment convention (lane l, g = l / 32): the A operand is A[l % 32][k0 + g], the B operand
// B[k0 + g][l % 32] for the two k values k0, k0 + 1 of one instruction; of the 16 results, value v
// belongs to row 8 (v / 4) + 4 g + v % 4, column l % 32.
#include "gta_internal.h"

namespace gta {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kCols = 64;                   // columns of Y per workgroup
constexpr int kChunk = 16;                  // k values of X staged at a time
constexpr int kStagePitch = kChunk + 1;     // floats; odd, so the 32 rows of a fragment read hit 32 banks
constexpr int kPatchPitch = kCols + 4;      // floats; rows stay 16-byte aligned

__device__ __forceinline__ void wave_lds_fence() {   // orders LDS traffic between the lanes of one wavefront
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

inline size_t linear_f32_lds_bytes(int d_in) {
    return sizeof(float) * ((size_t)kCols * (d_in + 1) + (size_t)(kThreads / 64) * 32 * kPatchPitch);
}

// Y[n, d_out] = X[n, d_in] * op(W) (+ C).  Workgroup b: column tile b % col_tiles, row tiles
// b / col_tiles, then every (gridDim.x / col_tiles)-th.  Every access is bounds-checked (rows
// past the end are read from the last row and never stored).
template <bool W_KMAJOR>
__global__ void __launch_bounds__(kThreads)
k_linear_f32(const float* __restrict__ X, const float* __restrict__ W, const float* C, float* Y, int64_t n,
             int d_in, int d_out, int col_tiles, int64_t row_tiles) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    float* panel = reinterpret_cast<float*>(lds_raw);   // [64][d_in + 1]: op(W)'s columns, k contiguous
    const int pitch = d_in + 1;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 5, r32 = lane & 31;
    float* patch = panel + kCols * pitch + w * 32 * kPatchPitch;   // this wavefront's [32][kPatchPitch]
    float* stage = patch;                                          // its X stage [32][kStagePitch] shares the space
    const int col0 = (int)(blockIdx.x % col_tiles) * kCols;
    const int64_t first_tile = blockIdx.x / col_tiles, tile_stride = gridDim.x / col_tiles;

    if (W_KMAJOR) {   // W [d_out, d_in]: rows are copied
        const int quads = d_in / 4;
        for (int u = threadIdx.x; u < kCols * quads; u += kThreads) {
            const int c = u / quads, kq = u - c * quads;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (col0 + c < d_out) v = *reinterpret_cast<const float4*>(W + (int64_t)(col0 + c) * d_in + 4 * kq);
            float* dst = panel + c * pitch + 4 * kq;
            dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
        }
    } else {          // W [d_in, d_out]: transposed while staged
        for (int u = threadIdx.x; u < d_in * (kCols / 4); u += kThreads) {
            const int k = u / (kCols / 4), cq = u - k * (kCols / 4);
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (col0 + 4 * cq < d_out) v = *reinterpret_cast<const float4*>(W + (int64_t)k * d_out + col0 + 4 * cq);
            float* dst = panel + (4 * cq) * pitch + k;
            dst[0] = v.x; dst[pitch] = v.y; dst[2 * pitch] = v.z; dst[3 * pitch] = v.w;
        }
    }
    __syncthreads();   // the only workgroup-wide synchronisation

    const int urow = lane >> 2, ucol = lane & 3;   // X chunk: 2 loads of 16 rows x 16 floats, a float4 per lane
    const int chunks = d_in / kChunk;
    for (int64_t tile = first_tile; tile < row_tiles; tile += tile_stride) {
        const int64_t row0 = tile * 128 + 32 * w;
        if (row0 >= n) continue;   // uniform over the wavefront; no workgroup barrier below
        auto fetch = [&](float4 (&dst)[2], int c) {
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                int64_t row = row0 + 16 * q + urow;
                if (row >= n) row = n - 1;
                dst[q] = *reinterpret_cast<const float4*>(X + row * d_in + c * kChunk + 4 * ucol);
            }
        };
        floatx16 acc[2];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
        float4 cur[2], nxt[2];
        fetch(cur, 0);
        for (int c = 0; c < chunks; ++c) {
            wave_lds_fence();   // earlier reads of the stage / patch by this wavefront are issued
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                float* dst = stage + (16 * q + urow) * kStagePitch + 4 * ucol;
                dst[0] = cur[q].x; dst[1] = cur[q].y; dst[2] = cur[q].z; dst[3] = cur[q].w;
            }
            if (c + 1 < chunks) fetch(nxt, c + 1);   // in flight during this chunk's arithmetic
            wave_lds_fence();
            const float* xrow = stage + r32 * kStagePitch + g;
            const float* wrow = panel + r32 * pitch + c * kChunk + g;
#pragma unroll
            for (int k0 = 0; k0 < kChunk; k0 += 2) {
                const float xb = xrow[k0];
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(wrow[32 * t * pitch + k0], xb, acc[t], 0, 0, 0);
            }
            cur[0] = nxt[0];
            cur[1] = nxt[1];
        }
        // acc[t][v]: row r32, column 32 t + 8 (v / 4) + 4 g + v % 4 of the 32 x 64 tile
        float* mine = patch + r32 * kPatchPitch + 4 * g;
        if (C) {
            wave_lds_fence();
#pragma unroll
            for (int q = 0; q < 8; ++q) {   // 32 rows x 16 units of 4 columns, coalesced
                const int u = lane + 64 * q, r = u >> 4, cu = u & 15;
                float4 cv = make_float4(0.f, 0.f, 0.f, 0.f);
                if (row0 + r < n && col0 + 4 * cu < d_out)
                    cv = *reinterpret_cast<const float4*>(C + (row0 + r) * d_out + col0 + 4 * cu);
                *reinterpret_cast<float4*>(patch + r * kPatchPitch + 4 * cu) = cv;
            }
            wave_lds_fence();
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    const float4 cv = *reinterpret_cast<const float4*>(mine + 32 * t + 8 * qd);
                    acc[t][4 * qd + 0] += cv.x; acc[t][4 * qd + 1] += cv.y;
                    acc[t][4 * qd + 2] += cv.z; acc[t][4 * qd + 3] += cv.w;
                }
        }
        wave_lds_fence();
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int qd = 0; qd < 4; ++qd)
                *reinterpret_cast<float4*>(mine + 32 * t + 8 * qd) =
                    make_float4(acc[t][4 * qd + 0], acc[t][4 * qd + 1], acc[t][4 * qd + 2], acc[t][4 * qd + 3]);
        wave_lds_fence();
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int u = lane + 64 * q, r = u >> 4, cu = u & 15;
            if (row0 + r < n && col0 + 4 * cu < d_out)
                *reinterpret_cast<float4*>(Y + (row0 + r) * d_out + col0 + 4 * cu) =
                    *reinterpret_cast<const float4*>(patch + r * kPatchPitch + 4 * cu);
        }
    }
}

// dW[d_in, d_out] = X^T dY over one block of rows: 128 x 128 tile per workgroup, wavefront
// (w / 2, w % 2) owns a 64 x 64 quarter.  The reduction index is the row, so 16-row blocks of both
// operands are staged row-major and fragments are plain 4-byte reads along a row (consecutive
// lanes, consecutive columns).  Row blocks are summed afterwards in a fixed order.
constexpr int kDwRows = 16, kDwPitch = 128 + 4;

__global__ void __launch_bounds__(kThreads)
k_linear_dw_f32(const float* __restrict__ X, const float* __restrict__ dY, float* __restrict__ partial, int64_t n,
                int d_in, int d_out, int64_t rows_per_split, int tiles_i, int tiles_o, int splits) {
    __shared__ __align__(16) float xs[kDwRows * kDwPitch], ys[kDwRows * kDwPitch];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 5, r32 = lane & 31;
    const int64_t bid = blockIdx.x, jj = bid >> 3;   // tiles of one row split get ids 8 apart (same XCD)
    const int tiles = tiles_i * tiles_o;
    const int tile = (int)(jj % tiles);
    const int64_t split = (jj / tiles) * 8 + (bid & 7);
    if (split >= splits) return;   // whole workgroup leaves together
    const int i0 = (tile % tiles_i) * 128, o0 = (tile / tiles_i) * 128;
    const int64_t rbeg = split * rows_per_split;
    const int64_t rend = rbeg + rows_per_split < n ? rbeg + rows_per_split : n;
    const int wi = w >> 1, wo = w & 1;

    // loader role: threads 0..127 stage X, 128..255 stage dY; a thread takes one row, 4 float4 32 columns apart
    const bool loads_x = threadIdx.x < 128;
    const int lt = threadIdx.x & 127, lrow = lt >> 3, lcol = 4 * (lt & 7);
    const float* src = loads_x ? X : dY;
    const int ld = loads_x ? d_in : d_out;
    const int cbase = (loads_x ? i0 : o0) + lcol;
    float* dst = (loads_x ? xs : ys) + lrow * kDwPitch + lcol;
    auto fetch = [&](float4 (&slot)[4], int64_t r0) {
        const int64_t r = r0 + lrow;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            slot[q] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (r < rend && cbase + 32 * q < ld) slot[q] = *reinterpret_cast<const float4*>(src + r * ld + cbase + 32 * q);
        }
    };

    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    float4 cur[4], nxt[4];
    fetch(cur, rbeg);
    for (int64_t r0 = rbeg; r0 < rend; r0 += kDwRows) {   // uniform over the workgroup
        __syncthreads();   // the previous block's fragments have been read
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<float4*>(dst + 32 * q) = cur[q];
        __syncthreads();
        fetch(nxt, r0 + kDwRows);   // all zeros past the end
#pragma unroll
        for (int k0 = 0; k0 < kDwRows; k0 += 2) {
            float af[2], bf[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                af[t] = xs[(k0 + g) * kDwPitch + 64 * wi + 32 * t + r32];
                bf[t] = ys[(k0 + g) * kDwPitch + 64 * wo + 32 * t + r32];
            }
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[a], bf[b], acc[a][b], 0, 0, 0);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) cur[q] = nxt[q];
    }
    float* out = partial + split * d_in * d_out;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int o = o0 + 64 * wo + 32 * b + r32;
            if (o >= d_out) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = i0 + 64 * wi + 32 * a + 8 * (v / 4) + 4 * g + v % 4;
                if (i < d_in) out[(int64_t)i * d_out + o] = acc[a][b][v];
            }
        }
}

}  // namespace

gta_status launch_linear_f32(const float* X, const float* W, const float* C, float* Y, int64_t n, int d_in,
                             int d_out, int trans_w, hipStream_t st) {
    const size_t lds = linear_f32_lds_bytes(d_in);
    if (lds > 160 * 1024) return fail(GTA_ERR_UNSUPPORTED, "fp32: d_in <= 496 is supported (the weight panel must fit in LDS)");
    const int col_tiles = (d_out + kCols - 1) / kCols;
    const int64_t row_tiles = (n + 127) / 128;
    int64_t row_groups = 1024 / col_tiles;   // about 4 workgroups per compute unit when LDS allows
    if (row_groups < 1) row_groups = 1;
    if (row_groups > row_tiles) row_groups = row_tiles;
    const int64_t blocks = row_groups * col_tiles;
    LaunchTimer t(trans_w ? "linear_nt" : "linear_nn", n, 0, st);
    if (trans_w) {
        GTA_HIP_TRY(hipFuncSetAttribute((const void*)k_linear_f32<true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(k_linear_f32<true>, dim3((unsigned)blocks), dim3(kThreads), lds, st, X, W, C, Y, n, d_in,
                           d_out, col_tiles, row_tiles);
    } else {
        GTA_HIP_TRY(hipFuncSetAttribute((const void*)k_linear_f32<false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(k_linear_f32<false>, dim3((unsigned)blocks), dim3(kThreads), lds, st, X, W, C, Y, n, d_in,
                           d_out, col_tiles, row_tiles);
    }
    GTA_HIP_TRY(hipGetLastError());
    return GTA_OK;
}

void launch_linear_dw_f32(const float* X, const float* dY, float* partial, int64_t n, int d_in, int d_out,
                          int64_t rows_per_split, int tiles_i, int tiles_o, int splits, hipStream_t st) {
    const int64_t blocks = (int64_t)(splits + 7) / 8 * 8 * tiles_i * tiles_o;
    hipLaunchKernelGGL(k_linear_dw_f32, dim3((unsigned)blocks), dim3(kThreads), 0, st, X, dY, partial, n, d_in, d_out,
                       rows_per_split, tiles_i, tiles_o, splits);
}

}  // namespace gta
