// Internal declarations shared by the translation units of libgta (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>

#include "gta.h"

#define GTA_API __attribute__((visibility("default")))

namespace gta {

// One side of the plan: the rows of a CSR pattern (destination rows of A, or source rows of
// A^T) ordered for scheduling.
struct Side {
    int64_t n_rows = 0;
    const int64_t* ptr = nullptr;   // device: row pointer of this side's pattern
    const int32_t* idx = nullptr;   // device: column ids (the other side's rows)
    int32_t* bin_rows = nullptr;    // device [n_rows]
    int2* span = nullptr;           // device [n_rows]: (ptr[row], ptr[row + 1]) of bin_rows[r], so a kernel
                                    // can fetch a row's id and its extent in one step instead of two
    int32_t* chunk_ptr = nullptr;   // device [n_chunked + 1]
    int4* chunks = nullptr;         // device [n_chunks] = (row, begin, end, chunks of row)
    int64_t bin_off[GTA_NUM_CLASSES + 1] = {0};   // host copy
    int64_t class_entries[GTA_NUM_CLASSES] = {0}; // host: stored entries per degree class (key order)
    int64_t n_chunked = 0, n_hub = 0, n_chunks = 0;
    int64_t n_hub_chunks = 0;       // chunks of the n_hub rows cut into several chunks: chunks[0 .. n_hub_chunks), the
                                    // only ones that leave partial results
};

}  // namespace gta

struct gta_plan {
    int64_t n_dst = 0, n_src = 0, nnz = 0;
    int32_t pack_max_deg = 0, wave_max_deg = 0, hub_chunk = 0;
    int64_t keep_dz_min_nnz = 262144;
    int device = 0;
    char* workspace = nullptr;     // device: base of the caller's buffer that holds every plan array
    size_t retained_bytes = 0;     // its leading part that stays in use after the plan is built
    const int64_t* indptr = nullptr;
    const int32_t* indices = nullptr;
    int64_t* t_indptr = nullptr;   // device [n_src + 1]
    int32_t* t_indices = nullptr;  // device [nnz]
    int32_t* t_eid = nullptr;      // device [nnz]: stored position of each transposed entry
    int32_t* t_pos = nullptr;      // device [nnz]: inverse of t_eid (transposed position of each stored entry)
    gta::Side side[2];
};

namespace gta {

// ---- error plumbing -------------------------------------------------------------------
gta_status fail(gta_status code, const char* fmt, ...);
#define GTA_HIP_TRY(expr)                                                                     \
    do {                                                                                      \
        hipError_t _e = (expr);                                                               \
        if (_e != hipSuccess)                                                                 \
            return ::gta::fail(GTA_ERR_HIP, "%s failed: %s (%s:%d)", #expr,                   \
                               hipGetErrorString(_e), __FILE__, __LINE__);                    \
    } while (0)

// degree class of a row and the sort key that orders rows hubs-first
__host__ __device__ inline int degree_class(int64_t deg) {
    if (deg <= 0) return 0;
    int bits = 0;
    for (uint64_t t = (uint64_t)(deg - 1); t; t >>= 1) ++bits;
    return 1 + bits;
}
inline int class_key(int cls) { return (GTA_NUM_CLASSES - 1) - cls; }

// ---- per-launch timing ------------------------------------------------------------------
struct LaunchTimer {   // RAII: records events around one launch when profiling is on
    LaunchTimer(const char* name, int64_t rows, int64_t entries, hipStream_t stream);
    ~LaunchTimer();
    int slot;
    hipStream_t stream;
};

bool split_launches();   // true while per-schedule timing (profile mode 2) is requested

// ---- shape handling ---------------------------------------------------------------------
struct Shape {
    int heads, head_dim, elem_bytes;   // heads = all heads of a row (the stride of per-head arrays)
    int head_bytes;
    int slice_heads, n_slices;   // a row is processed in n_slices launches of slice_heads heads each
    int lanes_per_head;   // LH: 16-byte lanes covering one head
    int lanes_per_row;    // G : 16-byte lanes covering one slice of a row (slice_heads * LH)
    int nv;               // values per lane (4 fp32, 8 bf16)
    int64_t row_bytes;    // all heads: the row stride
};
gta_status make_shape(int heads, int head_dim, gta_dtype dtype, Shape* out);

// Which rows go to which schedule, resolved from the plan for a given lanes_per_row.
struct Split {
    int64_t chunk_rows;            // bin_rows[0 .. chunk_rows)           -> chunk schedule
    int64_t wave_begin, wave_end;  // bin_rows[wave_begin .. wave_end)    -> one wavefront per row
    int64_t pack_begin, pack_end;  // bin_rows[pack_begin .. pack_end)    -> several rows per wavefront
    int64_t wave_entries, pack_entries, chunk_entries;
};
Split make_split(const gta_plan* plan, int side, int lanes_per_row);

// arguments common to the attention launches
// A tensor with one row per source that may live in two allocations (Algorithm 1: the rows this
// GPU owns, then the halo rows it received): rows below the split are in `lo`, the others in
// `hi`, which is kept pre-offset by -split rows so that both are addressed with the source id.
struct SegConst { const char *lo, *hi; };
struct SegMut { char *lo, *hi; };

struct AttnArgs {
    const gta_plan* plan;
    const void *Q, *K, *V, *out, *dO;
    void *o_out, *dQ, *dK, *dV;
    const void *K_halo, *V_halo;   // rows n_local .. n_src-1 of K / V when they are separate, else null
    void *dK_halo, *dV_halo;       // ... and of dK / dV
    int64_t n_local;               // meaningful when K_halo is set
    const float* lse_in;
    float* lse_out;
    float2* rowstat;     // [n_dst, heads] (lse * log2(e), delta)
    float* partial;      // scratch for split rows
    float* dS;           // [nnz, heads] softmax-backward values per stored entry, or null
    float scale;
    Shape shape;
    hipStream_t stream;
};

AttnArgs slice_args(const AttnArgs& a, int slice);   // pointers moved to the slice's first head

inline int seg_split(const AttnArgs& a) { return a.K_halo ? (int)a.n_local : INT32_MAX; }
inline SegConst seg_of(const AttnArgs& a, const void* local, const void* halo) {
    const char* lo = static_cast<const char*>(local);
    if (!a.K_halo) return SegConst{lo, lo};
    return SegConst{lo, reinterpret_cast<const char*>(reinterpret_cast<uintptr_t>(halo) -
                                                      (uintptr_t)(a.n_local * a.shape.row_bytes))};
}
inline SegMut seg_of(const AttnArgs& a, void* local, void* halo) {
    char* lo = static_cast<char*>(local);
    if (!a.K_halo) return SegMut{lo, lo};
    return SegMut{lo, reinterpret_cast<char*>(reinterpret_cast<uintptr_t>(halo) -
                                              (uintptr_t)(a.n_local * a.shape.row_bytes))};
}

gta_status launch_fwd(const AttnArgs& a);
gta_status launch_bwd_dst(const AttnArgs& a);
gta_status launch_bwd_src(const AttnArgs& a);   // stores dS when a.dS is set
gta_status launch_rowstat(const AttnArgs& a);   // (lse * log2 e, dY_i . Y_i) per (row, head)
gta_status launch_bwd_dq(const AttnArgs& a);    // dQ = scale * dS K over the stored dS

// grouped projections Y_po = sum_pi X_pi op(W[po][pi]) (+ C_po): bf16, d in {64, 128, 256}
bool proj_group_supported(int d, gta_dtype dtype);
size_t proj_group_scratch_bytes(int d, int mats);
gta_status proj_group(const void* const* X, int p_in, const void* const* W, int p_out, const void* const* C,
                      void* const* Y, int64_t n, int d, int trans_w, void* scratch, size_t scratch_bytes,
                      hipStream_t st);

// fp32 forms of the dense projections (the bf16 forms live with their entry points)
gta_status launch_linear_f32(const float* X, const float* W, const float* C, float* Y, int64_t n, int d_in,
                             int d_out, int trans_w, hipStream_t st);
void launch_linear_dw_f32(const float* X, const float* dY, float* partial, int64_t n, int d_in, int d_out,
                          int64_t rows_per_split, int tiles_i, int tiles_o, int splits, hipStream_t st);

}  // namespace gta
