// Scheduling plan: degree classes, hubs-first row order, chunk tables and the transposed
// pattern, all built on the GPU with integer-only kernels (stable LSD radix sort, prefix sums,
// binary searches).  The transposed pattern is what the backward's SpMMs with the transposed
// adjacency run over (paper Section 2.2: dV = U^T dY, dK = dZ^T Q); the stable order fixes
// their summation order.
#include "gta_internal.h"

#include <type_traits>

#include <algorithm>
#include <new>

namespace gta {
namespace {

constexpr int kSortThreads = 256;                 // 4 wavefronts
constexpr int kWaveItems = 2048;                  // keys one wavefront ranks, in order
constexpr int kScanTile = 2048;                   // 256 threads x 8

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }

// ------------------------------------------------------------------ elementwise helpers
__global__ void k_iota(int32_t* v, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) v[i] = (int32_t)i;
}

__global__ void k_invert(const int32_t* perm, int32_t* inv, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) inv[perm[i]] = (int32_t)i;
}

__global__ void k_copy_keys(const int32_t* in, uint32_t* out, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = (uint32_t)in[i];
}

// key = 32 - class(degree), value = row id; also per-class row and entry counts
__global__ void k_degree_keys(const int64_t* ptr, int64_t n, uint32_t* keys, int32_t* vals,
                              unsigned long long* stats /* [33] rows, then [33] entries */) {
    __shared__ unsigned long long s_rows[GTA_NUM_CLASSES], s_ent[GTA_NUM_CLASSES];
    for (int t = threadIdx.x; t < GTA_NUM_CLASSES; t += blockDim.x) { s_rows[t] = 0; s_ent[t] = 0; }
    __syncthreads();
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        int64_t deg = ptr[i + 1] - ptr[i];
        int key = (GTA_NUM_CLASSES - 1) - degree_class(deg);
        keys[i] = (uint32_t)key;
        vals[i] = (int32_t)i;
        atomicAdd(&s_rows[key], 1ull);
        atomicAdd(&s_ent[key], (unsigned long long)deg);
    }
    __syncthreads();
    for (int t = threadIdx.x; t < GTA_NUM_CLASSES; t += blockDim.x) {
        if (s_rows[t]) atomicAdd(&stats[t], s_rows[t]);
        if (s_ent[t]) atomicAdd(&stats[GTA_NUM_CLASSES + t], s_ent[t]);
    }
}

__global__ void k_validate(const int64_t* indptr, const int32_t* indices, int64_t n_dst,
                           int64_t n_src, int64_t nnz, int* bad) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0 && (indptr[0] != 0 || indptr[n_dst] != nnz)) atomicOr(bad, 1);
    if (i < n_dst && indptr[i + 1] < indptr[i]) atomicOr(bad, 2);
    if (i < nnz && (indices[i] < 0 || (int64_t)indices[i] >= n_src)) atomicOr(bad, 4);
}

// ------------------------------------------------------------------ stable radix pass
// Each wavefront owns kWaveItems consecutive keys.  hist is digit-major [256][n_waves] so that
// one exclusive prefix sum over the flat array yields every (digit, wavefront) start offset.
__global__ void __launch_bounds__(kSortThreads)
k_radix_hist(const uint32_t* keys, int64_t n, int shift, int32_t* hist, int64_t n_waves) {
    __shared__ int cnt[kSortThreads / 64][256];
    const int w = threadIdx.x >> 6, lane = lane_id();
    const int64_t gw = (int64_t)blockIdx.x * (kSortThreads / 64) + w;
    for (int d = lane; d < 256; d += 64) cnt[w][d] = 0;
    __syncthreads();
    if (gw < n_waves) {
        const int64_t base = gw * kWaveItems;
        for (int s = 0; s < kWaveItems / 64; ++s) {
            int64_t i = base + s * 64 + lane;
            if (i < n) atomicAdd(&cnt[w][(keys[i] >> shift) & 255u], 1);
        }
    }
    __syncthreads();
    if (gw < n_waves)
        for (int d = lane; d < 256; d += 64) hist[(int64_t)d * n_waves + gw] = cnt[w][d];
}

__global__ void __launch_bounds__(kSortThreads)
k_radix_scatter(const uint32_t* keys_in, const int32_t* vals_in, uint32_t* keys_out,
                int32_t* vals_out, int64_t n, int shift, const int32_t* offs, int64_t n_waves) {
    __shared__ int cnt[kSortThreads / 64][256];
    const int w = threadIdx.x >> 6, lane = lane_id();
    const int64_t gw = (int64_t)blockIdx.x * (kSortThreads / 64) + w;
    if (gw < n_waves)
        for (int d = lane; d < 256; d += 64) cnt[w][d] = offs[(int64_t)d * n_waves + gw];
    __syncthreads();
    if (gw >= n_waves) return;
    const int64_t base = gw * kWaveItems;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    for (int s = 0; s < kWaveItems / 64; ++s) {
        const int64_t i = base + s * 64 + lane;
        const bool valid = i < n;
        const uint32_t key = valid ? keys_in[i] : 0u;
        const int val = valid ? vals_in[i] : 0;
        const int d = (int)((key >> shift) & 255u);
        // lanes holding the same digit (among valid lanes)
        unsigned long long m = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const unsigned long long bal = __ballot((d >> b) & 1);
            m &= ((d >> b) & 1) ? bal : ~bal;
        }
        const int leader = __ffsll((long long)m) - 1;
        int start = 0;
        if (valid && lane == leader) start = atomicAdd(&cnt[w][d], __popcll(m));
        start = __shfl(start, leader);
        if (valid) {
            const int64_t pos = (int64_t)start + __popcll(m & lt_mask);
            keys_out[pos] = key;
            vals_out[pos] = val;
        }
    }
}

// ------------------------------------------------------------------ exclusive prefix sum (int32)
__device__ __forceinline__ int block_exclusive_scan(int v, int* total) {
    __shared__ int wave_sum[kSortThreads / 64];
    const int lane = lane_id(), w = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
    }
    if (lane == 63) wave_sum[w] = incl;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int k = 0; k < kSortThreads / 64; ++k) {
        if (k < w) before += wave_sum[k];
        all += wave_sum[k];
    }
    __syncthreads();
    *total = all;
    return before + incl - v;
}

__global__ void __launch_bounds__(kSortThreads)
k_scan_reduce(const int32_t* in, int64_t n, int32_t* tile_sum) {
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * 8;
    int acc = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k)
        if (base + k < n) acc += in[base + k];
    int total;
    block_exclusive_scan(acc, &total);
    if (threadIdx.x == 0) tile_sum[blockIdx.x] = total;
}

// single block: exclusive scan of tile sums in place, any length
__global__ void __launch_bounds__(kSortThreads) k_scan_spine(int32_t* tile_sum, int64_t n_tiles) {
    int carry = 0;
    for (int64_t base = 0; base < n_tiles; base += kSortThreads) {
        const int64_t i = base + threadIdx.x;
        const int v = i < n_tiles ? tile_sum[i] : 0;
        int total;
        const int ex = block_exclusive_scan(v, &total);
        if (i < n_tiles) tile_sum[i] = carry + ex;
        carry += total;
    }
}

__global__ void __launch_bounds__(kSortThreads)
k_scan_apply(const int32_t* in, int32_t* out, int64_t n, const int32_t* tile_off) {
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * 8;
    int v[8], acc = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        v[k] = base + k < n ? in[base + k] : 0;
        acc += v[k];
    }
    int total;
    int run = block_exclusive_scan(acc, &total) + tile_off[blockIdx.x];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        if (base + k < n) out[base + k] = run;
        run += v[k];
    }
}

// ------------------------------------------------------------------ transpose helpers
// t_indptr[j] = first position whose sorted key is >= j  (j = 0 .. n_src)
__global__ void k_lower_bounds(const uint32_t* sorted, int64_t nnz, int64_t n_src, int64_t* t_indptr) {
    int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j > n_src) return;
    int64_t lo = 0, hi = nnz;
    while (lo < hi) {
        int64_t mid = (lo + hi) >> 1;
        if ((int64_t)sorted[mid] < j) lo = mid + 1; else hi = mid;
    }
    t_indptr[j] = lo;
}

// destination row of every stored position: one wavefront per row writes the row id over the
// row's positions (coalesced) ...
__global__ void __launch_bounds__(256)
k_expand_rows(const int64_t* indptr, int64_t n_dst, int32_t* row_of_pos) {
    const int64_t row = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6;
    if (row >= n_dst) return;
    const int lane = threadIdx.x & 63;
    const int64_t b = indptr[row], e = indptr[row + 1];
    for (int64_t x = b + lane; x < e; x += 64) row_of_pos[x] = (int32_t)row;
}
// ... and each transposed entry picks up the row of its stored position
__global__ void k_row_of_entry(const int32_t* row_of_pos, const int32_t* t_eid, int64_t nnz, int32_t* t_indices) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < nnz) t_indices[p] = row_of_pos[t_eid[p]];
}

// extent of every row in plan order (positions fit in 32 bits)
__global__ void k_row_spans(const int64_t* ptr, const int32_t* bin_rows, int64_t n_rows, int2* span) {
    int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_rows) return;
    const int row = bin_rows[r];
    span[r] = make_int2((int)ptr[row], (int)ptr[row + 1]);
}

// ------------------------------------------------------------------ chunk tables
__global__ void k_chunk_count(const int64_t* ptr, const int32_t* bin_rows, int64_t n_chunked,
                              int hub_chunk, int32_t* cnt) {
    int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r > n_chunked) return;
    if (r == n_chunked) { cnt[r] = 0; return; }
    const int row = bin_rows[r];
    const int64_t deg = ptr[row + 1] - ptr[row];
    cnt[r] = (int32_t)((deg + hub_chunk - 1) / hub_chunk);
}

__global__ void k_chunk_fill(const int64_t* ptr, const int32_t* bin_rows, const int32_t* chunk_ptr,
                             int64_t n_chunked, int hub_chunk, int4* chunks) {
    int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_chunked) return;
    const int row = bin_rows[r];
    const int64_t b = ptr[row], e = ptr[row + 1];
    const int first = chunk_ptr[r], cnt = chunk_ptr[r + 1] - first;
    for (int c = 0; c < cnt; ++c) {
        const int64_t cb = b + (int64_t)c * hub_chunk;
        const int64_t ce = cb + hub_chunk < e ? cb + hub_chunk : e;
        chunks[first + c] = make_int4(row, (int)cb, (int)ce, cnt);
    }
}

// ------------------------------------------------------------------ host side
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }
inline dim3 grid_for(int64_t n, int threads) { return dim3((unsigned)std::max<int64_t>(1, ceil_div(n, threads))); }

// Entry positions are 32-bit in the kernels, whose loops step past a row's end by up to one
// workgroup's stride (256) before they stop: keep that sum representable.
constexpr int64_t kMaxNnz = (1ll << 31) - 1024;

struct Opts { int pack, wave, chunk, validate; int64_t keep_dz; };

bool resolve_opts(const gta_plan_opts* o, Opts* r) {
    r->pack = o && o->pack_max_deg > 0 ? o->pack_max_deg : 0;
    r->wave = o && o->wave_max_deg > 0 ? o->wave_max_deg : 128;
    r->chunk = o && o->hub_chunk > 0 ? o->hub_chunk : 2048;
    r->validate = o ? o->validate : 0;
    r->keep_dz = !o || o->keep_dz_min_nnz == 0 ? 262144 : (o->keep_dz_min_nnz < 0 ? INT64_MAX : o->keep_dz_min_nnz);
    auto pow2 = [](int v) { return v > 0 && (v & (v - 1)) == 0; };
    if (!pow2(r->wave) || !pow2(r->chunk) || r->chunk < r->wave) return false;
    if (r->pack != 0 && (!pow2(r->pack) || r->pack > r->wave)) return false;
    return true;
}

struct Layout {
    size_t bin_rows[2], span[2], chunk_ptr[2], chunks[2], t_indptr, t_indices, t_eid, t_pos;
    size_t retained, key_a, key_b, val_a, val_b, hist, tile_sum, stats, flag, total;
    int64_t max_chunked[2], max_chunks[2], sort_cap, hist_cap, tile_cap;
};

void make_layout(int64_t n_dst, int64_t n_src, int64_t nnz, const Opts& o, Layout* L) {
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t at = off; off = align_up(off + bytes); return at; };
    const int64_t n_rows[2] = {n_dst, n_src};
    for (int s = 0; s < 2; ++s) {
        L->max_chunked[s] = std::min<int64_t>(n_rows[s], nnz / ((int64_t)o.wave + 1));
        L->max_chunks[s] = nnz / o.chunk + L->max_chunked[s];
        L->bin_rows[s] = take(sizeof(int32_t) * (size_t)std::max<int64_t>(1, n_rows[s]));
        L->span[s] = take(sizeof(int2) * (size_t)std::max<int64_t>(1, n_rows[s]));
        L->chunk_ptr[s] = take(sizeof(int32_t) * (size_t)(L->max_chunked[s] + 1));
        L->chunks[s] = take(sizeof(int4) * (size_t)std::max<int64_t>(1, L->max_chunks[s]));
    }
    L->t_indptr = take(sizeof(int64_t) * (size_t)(n_src + 1));
    L->t_indices = take(sizeof(int32_t) * (size_t)std::max<int64_t>(1, nnz));
    L->t_eid = take(sizeof(int32_t) * (size_t)std::max<int64_t>(1, nnz));
    L->t_pos = take(sizeof(int32_t) * (size_t)std::max<int64_t>(1, nnz));
    L->retained = off;   // everything from here on is needed only while the plan is being built
    L->sort_cap = std::max<int64_t>(1, std::max(nnz, std::max(n_dst, n_src)));
    L->key_a = take(4 * (size_t)L->sort_cap);
    L->key_b = take(4 * (size_t)L->sort_cap);
    L->val_a = take(4 * (size_t)L->sort_cap);
    L->val_b = take(4 * (size_t)L->sort_cap);
    L->hist_cap = 256 * ceil_div(L->sort_cap, kWaveItems);
    L->hist_cap = std::max<int64_t>(L->hist_cap, L->max_chunked[0] + 1);
    L->hist_cap = std::max<int64_t>(L->hist_cap, L->max_chunked[1] + 1);
    L->hist = take(4 * (size_t)L->hist_cap);
    L->tile_cap = ceil_div(L->hist_cap, kScanTile) + 1;
    L->tile_sum = take(4 * (size_t)L->tile_cap);
    L->stats = take(sizeof(unsigned long long) * 2 * GTA_NUM_CLASSES);
    L->flag = take(sizeof(int));
    L->total = off;
}

struct Builder {
    char* ws;
    Layout L;
    hipStream_t st;
    template <class T> T* at(size_t off) const { return reinterpret_cast<T*>(ws + off); }

    // exclusive prefix sum of n int32 values (in -> out, may alias)
    gta_status scan(const int32_t* in, int32_t* out, int64_t n) {
        if (n <= 0) return GTA_OK;
        const int64_t tiles = ceil_div(n, kScanTile);
        int32_t* tile_sum = at<int32_t>(L.tile_sum);
        hipLaunchKernelGGL(k_scan_reduce, dim3((unsigned)tiles), dim3(kSortThreads), 0, st, in, n, tile_sum);
        hipLaunchKernelGGL(k_scan_spine, dim3(1), dim3(kSortThreads), 0, st, tile_sum, tiles);
        hipLaunchKernelGGL(k_scan_apply, dim3((unsigned)tiles), dim3(kSortThreads), 0, st, in, out, n, tile_sum);
        GTA_HIP_TRY(hipGetLastError());
        return GTA_OK;
    }

    // stable sort of (key, val) pairs on the low `bits` bits; result pointers returned
    gta_status radix_sort(int64_t n, int bits, uint32_t** keys, int32_t** vals) {
        uint32_t *ka = at<uint32_t>(L.key_a), *kb = at<uint32_t>(L.key_b);
        int32_t *va = at<int32_t>(L.val_a), *vb = at<int32_t>(L.val_b);
        *keys = ka;
        *vals = va;
        if (n <= 0) return GTA_OK;
        const int64_t n_waves = ceil_div(n, kWaveItems);
        const unsigned blocks = (unsigned)ceil_div(n_waves, kSortThreads / 64);
        int32_t* hist = at<int32_t>(L.hist);
        for (int shift = 0; shift < bits; shift += 8) {
            hipLaunchKernelGGL(k_radix_hist, dim3(blocks), dim3(kSortThreads), 0, st, ka, n, shift, hist, n_waves);
            gta_status s = scan(hist, hist, 256 * n_waves);
            if (s != GTA_OK) return s;
            hipLaunchKernelGGL(k_radix_scatter, dim3(blocks), dim3(kSortThreads), 0, st, ka, va, kb, vb,
                               n, shift, hist, n_waves);
            std::swap(ka, kb);
            std::swap(va, vb);
        }
        GTA_HIP_TRY(hipGetLastError());
        *keys = ka;
        *vals = va;
        return GTA_OK;
    }

    gta_status build_side(const gta_plan* plan, Side* sd, int s, const int64_t* ptr, const int32_t* idx,
                          int64_t n_rows) {
        sd->n_rows = n_rows;
        sd->ptr = ptr;
        sd->idx = idx;
        sd->bin_rows = at<int32_t>(L.bin_rows[s]);
        sd->span = at<int2>(L.span[s]);
        sd->chunk_ptr = at<int32_t>(L.chunk_ptr[s]);
        sd->chunks = at<int4>(L.chunks[s]);
        unsigned long long* stats = at<unsigned long long>(L.stats);
        GTA_HIP_TRY(hipMemsetAsync(stats, 0, sizeof(unsigned long long) * 2 * GTA_NUM_CLASSES, st));
        uint32_t* ka = at<uint32_t>(L.key_a);
        int32_t* va = at<int32_t>(L.val_a);
        if (n_rows > 0)
            hipLaunchKernelGGL(k_degree_keys, grid_for(n_rows, 256), dim3(256), 0, st, ptr, n_rows, ka, va, stats);
        uint32_t* ks;
        int32_t* vs;
        gta_status rc = radix_sort(n_rows, 8, &ks, &vs);
        if (rc != GTA_OK) return rc;
        if (n_rows > 0) {
            GTA_HIP_TRY(hipMemcpyAsync(sd->bin_rows, vs, sizeof(int32_t) * (size_t)n_rows,
                                       hipMemcpyDeviceToDevice, st));
            hipLaunchKernelGGL(k_row_spans, grid_for(n_rows, 256), dim3(256), 0, st, ptr, sd->bin_rows, n_rows, sd->span);
        }
        unsigned long long h_stats[2 * GTA_NUM_CLASSES];
        GTA_HIP_TRY(hipMemcpyAsync(h_stats, stats, sizeof(h_stats), hipMemcpyDeviceToHost, st));
        GTA_HIP_TRY(hipStreamSynchronize(st));
        sd->bin_off[0] = 0;
        for (int k = 0; k < GTA_NUM_CLASSES; ++k) {
            sd->bin_off[k + 1] = sd->bin_off[k] + (int64_t)h_stats[k];
            sd->class_entries[k] = (int64_t)h_stats[GTA_NUM_CLASSES + k];
        }
        // rows with degree > 2^w are the classes >= w + 2
        auto rows_above = [&](int threshold) {
            int w = 0;
            while ((1 << w) < threshold) ++w;
            const int first_key_excluded = class_key(w + 2) + 1;   // keys 0 .. class_key(w+2)
            return first_key_excluded <= 0 ? (int64_t)0 : sd->bin_off[std::min(first_key_excluded, GTA_NUM_CLASSES)];
        };
        sd->n_chunked = rows_above(plan->wave_max_deg);
        sd->n_hub = rows_above(plan->hub_chunk);
        if (sd->n_chunked > L.max_chunked[s])
            return fail(GTA_ERR_WORKSPACE, "internal: chunked-row bound exceeded");
        int32_t* cnt = at<int32_t>(L.hist);
        hipLaunchKernelGGL(k_chunk_count, grid_for(sd->n_chunked + 1, 256), dim3(256), 0, st, ptr,
                           sd->bin_rows, sd->n_chunked, plan->hub_chunk, cnt);
        rc = scan(cnt, sd->chunk_ptr, sd->n_chunked + 1);
        if (rc != GTA_OK) return rc;
        int32_t total = 0, hub_total = 0;
        GTA_HIP_TRY(hipMemcpyAsync(&total, sd->chunk_ptr + sd->n_chunked, sizeof(int32_t),
                                   hipMemcpyDeviceToHost, st));
        GTA_HIP_TRY(hipMemcpyAsync(&hub_total, sd->chunk_ptr + sd->n_hub, sizeof(int32_t),
                                   hipMemcpyDeviceToHost, st));
        GTA_HIP_TRY(hipStreamSynchronize(st));
        sd->n_chunks = total;
        sd->n_hub_chunks = hub_total;
        if (sd->n_chunks > L.max_chunks[s])
            return fail(GTA_ERR_WORKSPACE, "internal: chunk bound exceeded");
        if (sd->n_chunked > 0)
            hipLaunchKernelGGL(k_chunk_fill, grid_for(sd->n_chunked, 256), dim3(256), 0, st, ptr,
                               sd->bin_rows, sd->chunk_ptr, sd->n_chunked, plan->hub_chunk, sd->chunks);
        GTA_HIP_TRY(hipGetLastError());
        return GTA_OK;
    }
};

}  // namespace
}  // namespace gta

using namespace gta;

extern "C" GTA_API size_t gta_plan_workspace_bytes(int64_t n_dst, int64_t n_src, int64_t nnz,
                                           const gta_plan_opts* opts) {
    Opts o;
    if (n_dst < 0 || n_src < 0 || nnz < 0 || n_dst >= (1ll << 31) || n_src >= (1ll << 31) ||
        nnz > kMaxNnz || !resolve_opts(opts, &o))
        return 0;
    Layout L;
    make_layout(n_dst, n_src, nnz, o, &L);
    return L.total;
}

extern "C" GTA_API gta_status gta_plan_create(gta_plan** out, const int64_t* indptr, const int32_t* indices,
                                      int64_t n_dst, int64_t n_src, int64_t nnz,
                                      const gta_plan_opts* opts, void* workspace,
                                      size_t workspace_bytes, void* stream) {
    if (!out) return fail(GTA_ERR_INVALID_ARG, "plan out-pointer is null");
    *out = nullptr;
    if (!indptr || (!indices && nnz > 0) || !workspace)
        return fail(GTA_ERR_INVALID_ARG, "null pointer argument");
    if (n_dst < 0 || n_src < 0 || nnz < 0) return fail(GTA_ERR_INVALID_ARG, "negative size");
    if (n_dst >= (1ll << 31) || n_src >= (1ll << 31) || nnz > kMaxNnz)
        return fail(GTA_ERR_UNSUPPORTED, "n_dst and n_src must be below 2^31, nnz at most 2^31 - 1024");
    if (n_src < n_dst) return fail(GTA_ERR_INVALID_ARG, "n_src must be >= n_dst (owned rows come first)");
    Opts o;
    if (!resolve_opts(opts, &o))
        return fail(GTA_ERR_INVALID_ARG, "thresholds must be powers of two with pack <= wave <= hub_chunk");
    if (((uintptr_t)workspace & 255) != 0) return fail(GTA_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    Builder b;
    b.ws = static_cast<char*>(workspace);
    b.st = static_cast<hipStream_t>(stream);
    make_layout(n_dst, n_src, nnz, o, &b.L);
    if (workspace_bytes < b.L.total)
        return fail(GTA_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, b.L.total);

    gta_plan* p = new (std::nothrow) gta_plan();
    if (!p) return fail(GTA_ERR_INVALID_ARG, "out of host memory");
    struct Guard { gta_plan* p; ~Guard() { delete p; } } guard{p};
    p->n_dst = n_dst; p->n_src = n_src; p->nnz = nnz;
    p->pack_max_deg = o.pack; p->wave_max_deg = o.wave; p->hub_chunk = o.chunk;
    p->keep_dz_min_nnz = o.keep_dz;
    p->indptr = indptr; p->indices = indices;
    p->workspace = b.ws;
    p->retained_bytes = b.L.retained;
    GTA_HIP_TRY(hipGetDevice(&p->device));

    if (o.validate) {
        int* flag = b.at<int>(b.L.flag);
        GTA_HIP_TRY(hipMemsetAsync(flag, 0, sizeof(int), b.st));
        hipLaunchKernelGGL(k_validate, grid_for(std::max(n_dst, nnz) + 1, 256), dim3(256), 0, b.st,
                           indptr, indices, n_dst, n_src, nnz, flag);
        int h = 0;
        GTA_HIP_TRY(hipMemcpyAsync(&h, flag, sizeof(int), hipMemcpyDeviceToHost, b.st));
        GTA_HIP_TRY(hipStreamSynchronize(b.st));
        if (h) return fail(GTA_ERR_GRAPH, "malformed CSR (%s%s%s)", (h & 1) ? "indptr ends; " : "",
                           (h & 2) ? "indptr not monotone; " : "", (h & 4) ? "index out of range" : "");
    }

    // destination side: scheduling order of the rows of A
    gta_status rc = b.build_side(p, &p->side[0], 0, indptr, indices, n_dst);
    if (rc != GTA_OK) return rc;

    // transposed pattern: stable sort of stored positions by source id
    p->t_indptr = b.at<int64_t>(b.L.t_indptr);
    p->t_indices = b.at<int32_t>(b.L.t_indices);
    p->t_eid = b.at<int32_t>(b.L.t_eid);
    p->t_pos = b.at<int32_t>(b.L.t_pos);
    {
        uint32_t* ka = b.at<uint32_t>(b.L.key_a);
        int32_t* va = b.at<int32_t>(b.L.val_a);
        if (nnz > 0) {
            hipLaunchKernelGGL(k_copy_keys, grid_for(nnz, 256), dim3(256), 0, b.st, indices, ka, nnz);
            hipLaunchKernelGGL(k_iota, grid_for(nnz, 256), dim3(256), 0, b.st, va, nnz);
        }
        int bits = 1;
        while (bits < 32 && (1ll << bits) < n_src) ++bits;
        uint32_t* ks;
        int32_t* vs;
        rc = b.radix_sort(nnz, bits, &ks, &vs);
        if (rc != GTA_OK) return rc;
        hipLaunchKernelGGL(k_lower_bounds, grid_for(n_src + 1, 256), dim3(256), 0, b.st, ks, nnz, n_src, p->t_indptr);
        if (nnz > 0) {
            GTA_HIP_TRY(hipMemcpyAsync(p->t_eid, vs, sizeof(int32_t) * (size_t)nnz, hipMemcpyDeviceToDevice, b.st));
            // the sort's other value buffer is free now: it holds the row of every stored position
            int32_t* row_of_pos = vs == b.at<int32_t>(b.L.val_a) ? b.at<int32_t>(b.L.val_b) : b.at<int32_t>(b.L.val_a);
            hipLaunchKernelGGL(k_expand_rows, grid_for(n_dst * 64, 256), dim3(256), 0, b.st, indptr, n_dst, row_of_pos);
            hipLaunchKernelGGL(k_row_of_entry, grid_for(nnz, 256), dim3(256), 0, b.st, row_of_pos, p->t_eid, nnz,
                               p->t_indices);
            hipLaunchKernelGGL(k_invert, grid_for(nnz, 256), dim3(256), 0, b.st, p->t_eid, p->t_pos, nnz);
        }
        GTA_HIP_TRY(hipGetLastError());
    }

    // source side: scheduling order of the rows of A^T
    rc = b.build_side(p, &p->side[1], 1, p->t_indptr, p->t_indices, n_src);
    if (rc != GTA_OK) return rc;
    GTA_HIP_TRY(hipStreamSynchronize(b.st));
    guard.p = nullptr;
    *out = p;
    return GTA_OK;
}

extern "C" GTA_API size_t gta_plan_retained_bytes(int64_t n_dst, int64_t n_src, int64_t nnz, const gta_plan_opts* opts) {
    Opts o;
    if (n_dst < 0 || n_src < 0 || nnz < 0 || n_dst >= (1ll << 31) || n_src >= (1ll << 31) ||
        nnz > kMaxNnz || !resolve_opts(opts, &o))
        return 0;
    Layout L;
    make_layout(n_dst, n_src, nnz, o, &L);
    return L.retained;
}

extern "C" GTA_API gta_status gta_plan_compact(gta_plan* p, void* new_workspace, size_t new_bytes, void* stream) {
    if (!p || !new_workspace) return fail(GTA_ERR_INVALID_ARG, "null pointer argument");
    if (((uintptr_t)new_workspace & 255) != 0) return fail(GTA_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    if (new_bytes < p->retained_bytes)
        return fail(GTA_ERR_WORKSPACE, "the new workspace has %zu bytes, %zu needed", new_bytes, p->retained_bytes);
    int device = -1;
    GTA_HIP_TRY(hipGetDevice(&device));
    if (device != p->device)
        return fail(GTA_ERR_INVALID_ARG, "the plan lives on device %d, the current device is %d", p->device, device);
    char* to = static_cast<char*>(new_workspace);
    if (to == p->workspace) return GTA_OK;
    if (to < p->workspace + p->retained_bytes && p->workspace < to + p->retained_bytes)
        return fail(GTA_ERR_INVALID_ARG, "the new workspace overlaps the retained part of the old one");
    hipStream_t st = static_cast<hipStream_t>(stream);
    GTA_HIP_TRY(hipMemcpyAsync(to, p->workspace, p->retained_bytes, hipMemcpyDeviceToDevice, st));
    GTA_HIP_TRY(hipStreamSynchronize(st));
    const ptrdiff_t shift = to - p->workspace;
    auto move = [shift](auto*& ptr) {
        typedef std::remove_reference_t<decltype(ptr)> P;
        if (ptr) ptr = reinterpret_cast<P>(reinterpret_cast<char*>(const_cast<std::remove_const_t<std::remove_pointer_t<P>>*>(ptr)) + shift);
    };
    move(p->t_indptr); move(p->t_indices); move(p->t_eid); move(p->t_pos);
    for (int s = 0; s < 2; ++s) {
        Side& sd = p->side[s];
        move(sd.bin_rows); move(sd.span); move(sd.chunk_ptr); move(sd.chunks);
    }
    p->side[1].ptr = p->t_indptr;   // the source side walks the transposed pattern (the destination side the caller's CSR)
    p->side[1].idx = p->t_indices;
    p->workspace = to;
    return GTA_OK;
}

extern "C" GTA_API void gta_plan_destroy(gta_plan* plan) { delete plan; }

extern "C" GTA_API gta_status gta_plan_get_info(const gta_plan* p, gta_plan_info* info) {
    if (!p || !info) return fail(GTA_ERR_INVALID_ARG, "null pointer argument");
    info->n_dst = p->n_dst; info->n_src = p->n_src; info->nnz = p->nnz;
    info->pack_max_deg = p->pack_max_deg; info->wave_max_deg = p->wave_max_deg; info->hub_chunk = p->hub_chunk;
    for (int s = 0; s < 2; ++s) {
        info->n_chunked[s] = p->side[s].n_chunked;
        info->n_hub[s] = p->side[s].n_hub;
        info->n_chunks[s] = p->side[s].n_chunks;
    }
    return GTA_OK;
}

extern "C" GTA_API gta_status gta_plan_export_bins(const gta_plan* p, int side, int32_t* bin_rows,
                                           int64_t* bin_off, int32_t* chunk_ptr, int32_t* chunks) {
    if (!p || side < 0 || side > 1) return fail(GTA_ERR_INVALID_ARG, "bad plan or side");
    const Side& sd = p->side[side];
    GTA_HIP_TRY(hipDeviceSynchronize());
    if (bin_rows && sd.n_rows > 0)
        GTA_HIP_TRY(hipMemcpy(bin_rows, sd.bin_rows, sizeof(int32_t) * (size_t)sd.n_rows, hipMemcpyDeviceToHost));
    if (bin_off)
        for (int k = 0; k <= GTA_NUM_CLASSES; ++k) bin_off[k] = sd.bin_off[k];
    if (chunk_ptr)
        GTA_HIP_TRY(hipMemcpy(chunk_ptr, sd.chunk_ptr, sizeof(int32_t) * (size_t)(sd.n_chunked + 1), hipMemcpyDeviceToHost));
    if (chunks && sd.n_chunks > 0)
        GTA_HIP_TRY(hipMemcpy(chunks, sd.chunks, sizeof(int4) * (size_t)sd.n_chunks, hipMemcpyDeviceToHost));
    return GTA_OK;
}

extern "C" GTA_API gta_status gta_plan_export_transpose(const gta_plan* p, int64_t* t_indptr,
                                                int32_t* t_indices, int32_t* t_eid) {
    if (!p) return fail(GTA_ERR_INVALID_ARG, "plan is null");
    GTA_HIP_TRY(hipDeviceSynchronize());
    if (t_indptr)
        GTA_HIP_TRY(hipMemcpy(t_indptr, p->t_indptr, sizeof(int64_t) * (size_t)(p->n_src + 1), hipMemcpyDeviceToHost));
    if (t_indices && p->nnz > 0)
        GTA_HIP_TRY(hipMemcpy(t_indices, p->t_indices, sizeof(int32_t) * (size_t)p->nnz, hipMemcpyDeviceToHost));
    if (t_eid && p->nnz > 0)
        GTA_HIP_TRY(hipMemcpy(t_eid, p->t_eid, sizeof(int32_t) * (size_t)p->nnz, hipMemcpyDeviceToHost));
    return GTA_OK;
}
