// C ABI entry points, argument checking, shape / schedule resolution and launch timing.
#include "gta_internal.h"

#include <math.h>
#include <string.h>

#include <mutex>
#include <vector>

namespace gta {

// ---------------------------------------------------------------- errors
static thread_local char g_error[512] = "";

gta_status fail(gta_status code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof g_error, fmt, ap);
    va_end(ap);
    return code;
}

// ---------------------------------------------------------------- launch timing
namespace {
struct Record {
    char name[40];
    int64_t rows, entries;
    hipEvent_t a, b;
};
std::mutex g_prof_mutex;
std::vector<Record> g_records;
bool g_profiling = false;
bool g_split = false;
}  // namespace

bool split_launches() { return g_split; }

LaunchTimer::LaunchTimer(const char* name, int64_t rows, int64_t entries, hipStream_t st)
    : slot(-1), stream(st) {
    if (!g_profiling) return;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    Record r;
    memset(&r, 0, sizeof r);
    strncpy(r.name, name, sizeof r.name - 1);
    r.rows = rows;
    r.entries = entries;
    if (hipEventCreate(&r.a) != hipSuccess) return;
    if (hipEventCreate(&r.b) != hipSuccess) { (void)hipEventDestroy(r.a); return; }
    (void)hipEventRecord(r.a, st);
    g_records.push_back(r);
    slot = (int)g_records.size() - 1;
}
LaunchTimer::~LaunchTimer() {
    if (slot < 0) return;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (slot < (int)g_records.size()) (void)hipEventRecord(g_records[(size_t)slot].b, stream);
}

// ---------------------------------------------------------------- shapes and schedules
gta_status make_shape(int heads, int head_dim, gta_dtype dtype, Shape* out) {
    if (dtype != GTA_F32 && dtype != GTA_BF16) return fail(GTA_ERR_UNSUPPORTED, "unknown dtype %d", (int)dtype);
    if (heads <= 0 || head_dim <= 0) return fail(GTA_ERR_INVALID_ARG, "heads and head_dim must be positive");
    Shape s;
    s.heads = heads;
    s.head_dim = head_dim;
    s.elem_bytes = dtype == GTA_F32 ? 4 : 2;
    s.nv = 16 / s.elem_bytes;
    s.head_bytes = head_dim * s.elem_bytes;
    s.row_bytes = (int64_t)heads * s.head_bytes;
    const int hb = s.head_bytes;
    if (hb != 16 && hb != 32 && hb != 64 && hb != 128 && hb != 256)
        return fail(GTA_ERR_UNSUPPORTED, "head_dim*sizeof(element) = %d bytes; supported: 16, 32, 64, 128, 256", hb);
    s.lanes_per_head = hb / 16;
    // heads are taken slice_heads at a time: the largest power of two that divides `heads` and keeps
    // a slice within 1024 bytes (64 lanes of 16 bytes)
    int sh = 1;
    while (heads % (sh * 2) == 0 && (sh * 2) * hb <= 1024) sh *= 2;
    s.slice_heads = sh;
    s.n_slices = heads / sh;
    s.lanes_per_row = sh * s.lanes_per_head;
    if (s.lanes_per_row < 4)
        return fail(GTA_ERR_UNSUPPORTED, "heads=%d with %d-byte heads gives %d-byte slices; at least 64 bytes are needed",
                    heads, hb, sh * hb);
    *out = s;
    return GTA_OK;
}

AttnArgs slice_args(const AttnArgs& a, int slice) {
    AttnArgs b = a;
    const int h0 = slice * a.shape.slice_heads;
    const int64_t off = (int64_t)h0 * a.shape.head_bytes;
    auto mv = [off](const void* p) { return p ? static_cast<const void*>(static_cast<const char*>(p) + off) : nullptr; };
    auto mvw = [off](void* p) { return p ? static_cast<void*>(static_cast<char*>(p) + off) : nullptr; };
    b.Q = mv(a.Q); b.K = mv(a.K); b.V = mv(a.V); b.out = mv(a.out); b.dO = mv(a.dO);
    b.o_out = mvw(a.o_out); b.dQ = mvw(a.dQ); b.dK = mvw(a.dK); b.dV = mvw(a.dV);
    b.K_halo = mv(a.K_halo); b.V_halo = mv(a.V_halo); b.dK_halo = mvw(a.dK_halo); b.dV_halo = mvw(a.dV_halo);
    if (a.lse_in) b.lse_in = a.lse_in + h0;
    if (a.lse_out) b.lse_out = a.lse_out + h0;
    if (a.rowstat) b.rowstat = a.rowstat + h0;
    if (a.dS) b.dS = a.dS + h0;
    return b;
}

Split make_split(const gta_plan* plan, int side, int lanes_per_row) {
    const Side& sd = plan->side[side];
    const int W = 64 / lanes_per_row;
    Split sp;
    sp.chunk_rows = sd.n_chunked;
    int pack = plan->pack_max_deg > 0 ? plan->pack_max_deg : 4 * W;
    if (pack > plan->wave_max_deg) pack = plan->wave_max_deg;
    int64_t pack_begin = sd.n_rows;
    if (W > 1) {
        int p = 0;
        while ((2 << p) <= pack) ++p;            // largest power of two <= pack is 2^p
        const int key = class_key(p + 1);          // rows with degree <= 2^p are the classes <= p + 1
        pack_begin = sd.bin_off[key];
    }
    if (pack_begin < sd.n_chunked) pack_begin = sd.n_chunked;
    sp.wave_begin = sd.n_chunked;
    sp.wave_end = pack_begin;
    sp.pack_begin = pack_begin;
    sp.pack_end = sd.n_rows;
    sp.chunk_entries = sp.wave_entries = sp.pack_entries = 0;
    for (int k = 0; k < GTA_NUM_CLASSES; ++k) {
        const int64_t at = sd.bin_off[k];   // classes are contiguous, so the start decides the schedule
        if (sd.bin_off[k + 1] == at) continue;
        if (at < sd.n_chunked) sp.chunk_entries += sd.class_entries[k];
        else if (at < pack_begin) sp.wave_entries += sd.class_entries[k];
        else sp.pack_entries += sd.class_entries[k];
    }
    return sp;
}

namespace {

// rowstat | partial | dS.  `lean` ends before dS: enough for the forward and for the backward form
// that recomputes everything per entry; `total` also holds dS [nnz, heads] for the faster form.
struct ScratchLayout { size_t rowstat, partial, dS, lean, total; };

ScratchLayout scratch_layout(const gta_plan* plan, const Shape& sh) {
    ScratchLayout L;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t G = (size_t)sh.lanes_per_row, nv = (size_t)sh.nv;
    // only the chunks of rows cut into several chunks leave partial results (they come first)
    const size_t fwd = (size_t)plan->side[0].n_hub_chunks * G * (nv + 2);
    const size_t bsrc = (size_t)plan->side[1].n_hub_chunks * G * (2 * nv);
    L.rowstat = 0;
    L.partial = up(sizeof(float2) * (size_t)plan->n_dst * (size_t)sh.heads);
    L.dS = L.partial + up(sizeof(float) * (fwd > bsrc ? fwd : bsrc)) + 256;
    L.lean = L.dS;
    // Rows of up to 128 bytes (one cache line) never keep dZ: fetching an entry's dZ through the position
    // map costs about as much as a second row gather, so recomputing it from K and V is faster there
    // (measured on 128-byte rows: 17.4 against 17.9 ms per step) and needs no per-entry storage.
    const bool keeps_dz = (size_t)sh.slice_heads * (size_t)sh.head_bytes > 128;
    L.total = keeps_dz ? L.dS + up(sizeof(float) * (size_t)plan->nnz * (size_t)sh.heads) : L.lean;
    return L;
}

// the checks every call that takes a plan makes, apart from its scratch buffer
gta_status check_plan_call(const gta_plan* plan, const int64_t* indptr, const int32_t* indices, int64_t n_dst,
                           int64_t n_src, int heads, int head_dim, gta_dtype dtype, float* scale, Shape* sh) {
    if (!plan) return fail(GTA_ERR_INVALID_ARG, "plan is null");
    if (!indptr || (!indices && plan->nnz > 0)) return fail(GTA_ERR_INVALID_ARG, "null graph pointer");
    if (indptr != plan->indptr || indices != plan->indices)
        return fail(GTA_ERR_INVALID_ARG, "indptr/indices differ from the arrays the plan was built for");
    if (n_dst != plan->n_dst || n_src != plan->n_src)
        return fail(GTA_ERR_INVALID_ARG, "n_dst/n_src differ from the plan's (%lld, %lld)",
                    (long long)plan->n_dst, (long long)plan->n_src);
    int device = -1;
    GTA_HIP_TRY(hipGetDevice(&device));
    if (device != plan->device)
        return fail(GTA_ERR_INVALID_ARG, "the plan lives on device %d, the current device is %d", plan->device, device);
    gta_status rc = make_shape(heads, head_dim, dtype, sh);
    if (rc != GTA_OK) return rc;
    if (!(*scale > 0.f)) *scale = 1.0f / sqrtf((float)head_dim);
    return GTA_OK;
}

gta_status check_common(const gta_plan* plan, const int64_t* indptr, const int32_t* indices,
                        int64_t n_dst, int64_t n_src, int heads, int head_dim, gta_dtype dtype,
                        float* scale, void* scratch, size_t scratch_bytes, Shape* sh, ScratchLayout* sl) {
    const gta_status rc = check_plan_call(plan, indptr, indices, n_dst, n_src, heads, head_dim, dtype, scale, sh);
    if (rc != GTA_OK) return rc;
    *sl = scratch_layout(plan, *sh);
    if (!scratch) return fail(GTA_ERR_INVALID_ARG, "scratch is null");
    if (((uintptr_t)scratch & 255) != 0) return fail(GTA_ERR_INVALID_ARG, "scratch must be 256-byte aligned");
    if (scratch_bytes < sl->lean)
        return fail(GTA_ERR_WORKSPACE, "scratch has %zu bytes, at least %zu needed", scratch_bytes, sl->lean);
    return GTA_OK;
}

bool misaligned(const void* p) { return ((uintptr_t)p & 15) != 0; }

}  // namespace
}  // namespace gta

using namespace gta;

extern "C" GTA_API size_t gta_attn_scratch_bytes(const gta_plan* plan, int heads, int head_dim, gta_dtype dtype) {
    Shape sh;
    if (!plan || make_shape(heads, head_dim, dtype, &sh) != GTA_OK) return 0;
    return scratch_layout(plan, sh).total;
}

extern "C" GTA_API size_t gta_attn_scratch_bytes_min(const gta_plan* plan, int heads, int head_dim, gta_dtype dtype) {
    Shape sh;
    if (!plan || make_shape(heads, head_dim, dtype, &sh) != GTA_OK) return 0;
    return scratch_layout(plan, sh).lean;
}

namespace {

// K / V (and dK / dV) arrive either as one [n_src] tensor (halo pointers null) or as the first
// n_local rows plus a separate tensor with the remaining n_src - n_local rows.
gta_status check_halo(int64_t n_src, int64_t n_local, const void* a_halo, const void* b_halo) {
    if (n_local < 0 || n_local > n_src) return fail(GTA_ERR_INVALID_ARG, "n_local must be in [0, n_src]");
    if (n_local < n_src && (!a_halo || !b_halo)) return fail(GTA_ERR_INVALID_ARG, "null halo tensor pointer");
    if (misaligned(a_halo) || misaligned(b_halo))
        return fail(GTA_ERR_INVALID_ARG, "tensor base pointers must be 16-byte aligned");
    return GTA_OK;
}

// argument checks of the forward that do not concern the scratch buffer
gta_status check_fwd_tensors(const void* Q, const void* K, const void* V, const void* out, const float* lse,
                             int64_t n_dst, int64_t n_local) {
    if ((n_dst > 0 && (!Q || !out || !lse)) || (n_local > 0 && (!K || !V)))
        return fail(GTA_ERR_INVALID_ARG, "null tensor pointer");
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(out))
        return fail(GTA_ERR_INVALID_ARG, "tensor base pointers must be 16-byte aligned");
    return GTA_OK;
}

// launches the forward; `partial` receives the partial results of the rows cut into several chunks
gta_status run_fwd(const gta_plan* plan, const Shape& sh, const void* Q, const void* K, const void* V,
                   const void* K_halo, const void* V_halo, int64_t n_local, void* out, float* lse, int64_t n_src,
                   float scale, float* partial, void* stream) {
    AttnArgs a;
    memset(&a, 0, sizeof a);
    a.plan = plan; a.Q = Q; a.K = K; a.V = V; a.o_out = out; a.lse_out = lse;
    if (n_local < n_src) { a.K_halo = K_halo; a.V_halo = V_halo; a.n_local = n_local; }
    a.partial = partial;
    a.scale = scale; a.shape = sh; a.stream = static_cast<hipStream_t>(stream);
    for (int s = 0; s < sh.n_slices; ++s) {
        const gta_status rc = launch_fwd(slice_args(a, s));
        if (rc != GTA_OK) return rc;
    }
    return GTA_OK;
}

gta_status attn_fwd(const gta_plan* plan, const int64_t* indptr, const int32_t* indices, const void* Q,
                    const void* K, const void* V, const void* K_halo, const void* V_halo, int64_t n_local,
                    void* out, float* lse, int64_t n_dst, int64_t n_src, int heads, int head_dim,
                    gta_dtype dtype, float scale, void* scratch, size_t scratch_bytes, void* stream) {
    Shape sh;
    ScratchLayout sl;
    gta_status rc = check_common(plan, indptr, indices, n_dst, n_src, heads, head_dim, dtype, &scale,
                                 scratch, scratch_bytes, &sh, &sl);
    if (rc != GTA_OK) return rc;
    if ((rc = check_fwd_tensors(Q, K, V, out, lse, n_dst, n_local)) != GTA_OK) return rc;
    if (n_dst == 0) return GTA_OK;
    return run_fwd(plan, sh, Q, K, V, K_halo, V_halo, n_local, out, lse, n_src, scale,
                   reinterpret_cast<float*>(static_cast<char*>(scratch) + sl.partial), stream);
}

gta_status attn_bwd(const gta_plan* plan, const int64_t* indptr, const int32_t* indices, const void* Q,
                    const void* K, const void* V, const void* K_halo, const void* V_halo, int64_t n_local,
                    const void* out, const float* lse, const void* dOut, void* dQ, void* dK, void* dV,
                    void* dK_halo, void* dV_halo, int64_t n_dst, int64_t n_src, int heads, int head_dim,
                    gta_dtype dtype, float scale, void* scratch, size_t scratch_bytes, void* stream) {
    Shape sh;
    ScratchLayout sl;
    gta_status rc = check_common(plan, indptr, indices, n_dst, n_src, heads, head_dim, dtype, &scale,
                                 scratch, scratch_bytes, &sh, &sl);
    if (rc != GTA_OK) return rc;
    if ((n_dst > 0 && (!Q || !out || !lse || !dOut || !dQ)) || (n_local > 0 && (!K || !V || !dK || !dV)))
        return fail(GTA_ERR_INVALID_ARG, "null tensor pointer");
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(out) || misaligned(dOut) ||
        misaligned(dQ) || misaligned(dK) || misaligned(dV))
        return fail(GTA_ERR_INVALID_ARG, "tensor base pointers must be 16-byte aligned");
    AttnArgs a;
    memset(&a, 0, sizeof a);
    a.plan = plan; a.Q = Q; a.K = K; a.V = V; a.out = out; a.dO = dOut; a.lse_in = lse;
    a.dQ = dQ; a.dK = dK; a.dV = dV;
    if (n_local < n_src) {
        a.K_halo = K_halo; a.V_halo = V_halo; a.dK_halo = dK_halo; a.dV_halo = dV_halo; a.n_local = n_local;
    }
    a.rowstat = reinterpret_cast<float2*>(static_cast<char*>(scratch) + sl.rowstat);
    a.partial = reinterpret_cast<float*>(static_cast<char*>(scratch) + sl.partial);
    a.scale = scale; a.shape = sh; a.stream = static_cast<hipStream_t>(stream);
    const bool keep_dz = sl.total > sl.lean && scratch_bytes >= sl.total && n_dst > 0 &&
                         plan->nnz >= plan->keep_dz_min_nnz;
    if (keep_dz) a.dS = reinterpret_cast<float*>(static_cast<char*>(scratch) + sl.dS);
    for (int s = 0; s < sh.n_slices; ++s) {
        const AttnArgs b = slice_args(a, s);
        if (keep_dz) {
            // dZ kept per stored entry: row statistics, then dK/dV (+ dZ), then dQ as an SpMM over K
            if ((rc = launch_rowstat(b)) != GTA_OK) return rc;
            if ((rc = launch_bwd_src(b)) != GTA_OK) return rc;
            if ((rc = launch_bwd_dq(b)) != GTA_OK) return rc;
        } else {
            if (n_dst > 0 && (rc = launch_bwd_dst(b)) != GTA_OK) return rc;
            if (n_src > 0 && (rc = launch_bwd_src(b)) != GTA_OK) return rc;
        }
    }
    return GTA_OK;
}

}  // namespace

extern "C" GTA_API gta_status gta_attn_fwd(const gta_plan* plan, const int64_t* indptr, const int32_t* indices,
                                   const void* Q, const void* K, const void* V, void* out, float* lse,
                                   int64_t n_dst, int64_t n_src, int heads, int head_dim,
                                   gta_dtype dtype, float scale, void* scratch, size_t scratch_bytes,
                                   void* stream) {
    return attn_fwd(plan, indptr, indices, Q, K, V, nullptr, nullptr, n_src, out, lse, n_dst, n_src, heads,
                    head_dim, dtype, scale, scratch, scratch_bytes, stream);
}

extern "C" GTA_API gta_status gta_attn_bwd(const gta_plan* plan, const int64_t* indptr, const int32_t* indices,
                                   const void* Q, const void* K, const void* V, const void* out,
                                   const float* lse, const void* dOut, void* dQ, void* dK, void* dV,
                                   int64_t n_dst, int64_t n_src, int heads, int head_dim,
                                   gta_dtype dtype, float scale, void* scratch, size_t scratch_bytes,
                                   void* stream) {
    return attn_bwd(plan, indptr, indices, Q, K, V, nullptr, nullptr, n_src, out, lse, dOut, dQ, dK, dV,
                    nullptr, nullptr, n_dst, n_src, heads, head_dim, dtype, scale, scratch, scratch_bytes, stream);
}

extern "C" GTA_API gta_status gta_attn_fwd_halo(const gta_plan* plan, const int64_t* indptr,
                                        const int32_t* indices, const void* Q, const void* K_local,
                                        const void* V_local, const void* K_halo, const void* V_halo,
                                        int64_t n_local, void* out, float* lse, int64_t n_dst, int64_t n_src,
                                        int heads, int head_dim, gta_dtype dtype, float scale, void* scratch,
                                        size_t scratch_bytes, void* stream) {
    const gta_status rc = check_halo(n_src, n_local, K_halo, V_halo);
    if (rc != GTA_OK) return rc;
    return attn_fwd(plan, indptr, indices, Q, K_local, V_local, K_halo, V_halo, n_local, out, lse, n_dst, n_src,
                    heads, head_dim, dtype, scale, scratch, scratch_bytes, stream);
}

extern "C" GTA_API gta_status gta_attn_bwd_halo(const gta_plan* plan, const int64_t* indptr,
                                        const int32_t* indices, const void* Q, const void* K_local,
                                        const void* V_local, const void* K_halo, const void* V_halo,
                                        int64_t n_local, const void* out, const float* lse, const void* dOut,
                                        void* dQ, void* dK_local, void* dV_local, void* dK_halo, void* dV_halo,
                                        int64_t n_dst, int64_t n_src, int heads, int head_dim, gta_dtype dtype,
                                        float scale, void* scratch, size_t scratch_bytes, void* stream) {
    gta_status rc = check_halo(n_src, n_local, K_halo, V_halo);
    if (rc != GTA_OK) return rc;
    if ((rc = check_halo(n_src, n_local, dK_halo, dV_halo)) != GTA_OK) return rc;
    return attn_bwd(plan, indptr, indices, Q, K_local, V_local, K_halo, V_halo, n_local, out, lse, dOut, dQ,
                    dK_local, dV_local, dK_halo, dV_halo, n_dst, n_src, heads, head_dim, dtype, scale, scratch,
                    scratch_bytes, stream);
}

// ---------------------------------------------------------------- forward without any allocation
// For callers that cannot allocate device memory and have none to pass for scratch: the partial
// results of the rows cut into several chunks go to a fixed array in the library's own device image.
// Every GPU holds its own copy of that array at its own address; the address is looked up once per
// device, with that device current, and kept.
namespace {
constexpr size_t kNoallocScratchBytes = GTA_NOALLOC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char g_noalloc_scratch[kNoallocScratchBytes];
std::mutex g_noalloc_mutex;
void* g_noalloc_ptr[kMaxDevices] = {nullptr};

// device address of g_noalloc_scratch on the current device (`device`)
gta_status noalloc_scratch(int device, void** out) {
    if (device < 0 || device >= kMaxDevices)
        return fail(GTA_ERR_UNSUPPORTED, "device id %d is outside the supported range 0..%d", device, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_noalloc_mutex);
    if (!g_noalloc_ptr[device]) {
        void* ptr = nullptr;
        GTA_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_noalloc_scratch)));
        if (!ptr) return fail(GTA_ERR_HIP, "hipGetSymbolAddress returned a null address");
        g_noalloc_ptr[device] = ptr;
    }
    *out = g_noalloc_ptr[device];
    return GTA_OK;
}
}  // namespace

extern "C" GTA_API gta_status gta_attn_fwd_noalloc(const gta_plan* plan, const int64_t* indptr,
                                           const int32_t* indices, const void* Q, const void* K, const void* V,
                                           void* out, float* lse, int64_t n_dst, int64_t n_src, int heads,
                                           int head_dim, gta_dtype dtype, float scale, void* stream) {
    Shape sh;
    gta_status rc = check_plan_call(plan, indptr, indices, n_dst, n_src, heads, head_dim, dtype, &scale, &sh);
    if (rc != GTA_OK) return rc;
    if ((rc = check_fwd_tensors(Q, K, V, out, lse, n_dst, n_src)) != GTA_OK) return rc;
    const size_t need = sizeof(float) * (size_t)plan->side[0].n_hub_chunks * (size_t)sh.lanes_per_row *
                        (size_t)(sh.nv + 2);
    if (need > kNoallocScratchBytes)
        return fail(GTA_ERR_WORKSPACE,
                    "the rows cut into several chunks need %zu bytes of partial results; the built-in scratch "
                    "holds %zu (use gta_attn_fwd with caller-provided scratch)", need, kNoallocScratchBytes);
    if (n_dst == 0) return GTA_OK;
    void* partial = nullptr;
    if ((rc = noalloc_scratch(plan->device, &partial)) != GTA_OK) return rc;   // plan->device is current
    return run_fwd(plan, sh, Q, K, V, nullptr, nullptr, n_src, out, lse, n_src, scale,
                   static_cast<float*>(partial), stream);
}

extern "C" GTA_API gta_status gta_profile_enable(int on) {
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    g_profiling = on != 0;
    g_split = on == 2;
    return GTA_OK;
}

extern "C" GTA_API int gta_profile_read(gta_launch_record* out, int cap, int reset) {
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    const int n = (int)g_records.size();
    for (int i = 0; i < n; ++i) {
        Record& r = g_records[(size_t)i];
        (void)hipEventSynchronize(r.b);
        if (out && i < cap) {
            memcpy(out[i].name, r.name, sizeof r.name);
            out[i].ms = 0.f;
            (void)hipEventElapsedTime(&out[i].ms, r.a, r.b);
            out[i].rows = r.rows;
            out[i].entries = r.entries;
        }
    }
    if (reset) {
        for (Record& r : g_records) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
        g_records.clear();
    }
    return n;
}

extern "C" GTA_API const char* gta_last_error(void) { return g_error; }
extern "C" GTA_API const char* gta_version(void) { return "gta 0.1 (gfx950)"; }
