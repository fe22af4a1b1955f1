// The paper's operators as standalone kernels (Section 2.2 counts them: forward 1 SDDMM + softmax
// + 1 SpMM; backward 3 SpMM + 1 SDDMM), with the per-entry matrices Z, U, dU, dZ stored as
// float [nnz, heads].  They reuse the row schedules of the fused passes.  The fused path never
// calls them; they exist so the unfused decomposition can be run and timed operator by operator.
#include "gta_kernels.h"
#include "gta_spmm_pass.h"

#include <type_traits>

namespace gta {
namespace {

// ---------------------------------------------------------------- SDDMM: Z[e,h] = x_i . y_j
template <class T, int LH_, int G_>
struct SddmmPass {
    static constexpr int LH = LH_, G = G_, U = UnrollFor<G_>::value;
    static constexpr int NV = Elt<T>::NV;
    static constexpr bool kUsesEntryId = true;
    static constexpr int N = 1;   // nothing is accumulated across entries
    struct Params {
        const char *X, *Y;
        float* Z;
        float* partial;
        int64_t stride;
        int heads;
    };
    float x[NV];
    float f[N];
    uint4 yr[U];
    int eids[U];

    __device__ __forceinline__ void init(const Params& p, int row, int lig, bool active, bool) {
#pragma unroll
        for (int i = 0; i < NV; ++i) x[i] = 0.f;
        f[0] = 0.f;
        zp = p.Z;
        heads = p.heads;
        my_lig = lig;
        if (active) Elt<T>::unpack(load16(p.X, row, p.stride, lig), x);
    }
    __device__ __forceinline__ void load(const Params& p, int u, int j, int e, bool ok, int lig) {
        yr[u] = make_uint4(0, 0, 0, 0);
        eids[u] = e;
        if (ok) yr[u] = load16(p.Y, j, p.stride, lig);
    }
    __device__ __forceinline__ void compute(const bool (&ok)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float y[NV];
            Elt<T>::unpack(yr[u], y);
            float d = 0.f;
#pragma unroll
            for (int i = 0; i < NV; ++i) d = fmaf(x[i], y[i], d);
            d = head_allreduce<LH>(d);
            if (ok[u] && my_lig % LH == 0) zp[(int64_t)eids[u] * heads + my_lig / LH] = d;
        }
    }
    static __device__ __forceinline__ void combine(float (&)[N], const float (&)[N]) {}
    static __device__ __forceinline__ void finish(const Params&, int, int, const float (&)[N]) {}
    float* zp;
    int heads, my_lig;
};

// ---------------------------------------------------------------- edge softmax over float [nnz, H]
// A team of TEAM threads owns one row; thread t of the team walks the row's deg*H contiguous
// values with stride TEAM, so it always sees head t % H (TEAM is a multiple of H).
template <int TEAM> struct TeamReduce {
    // combines (m, l) pairs of an online softmax over the team members that share t % H
    static __device__ __forceinline__ void softmax(float& m, float& l, int H, float* lds) {
        for (int off = H; off < (TEAM < 64 ? TEAM : 64); off <<= 1) {
            const float om = __shfl_xor(m, off), ol = __shfl_xor(l, off);
            const float mn = fmaxf(m, om);
            l = l * fast_exp2(m - mn) + ol * fast_exp2(om - mn);
            m = mn;
        }
        if (TEAM > 64) {   // wavefronts of a workgroup: through LDS, in wavefront order
            const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
            __syncthreads();
            if (lane < H) { lds[(w * 64 + lane) * 2] = m; lds[(w * 64 + lane) * 2 + 1] = l; }
            __syncthreads();
            float am = kNegBig, al = 0.f;
            for (int k = 0; k < TEAM / 64; ++k) {
                const float om = lds[(k * 64 + lane % H) * 2], ol = lds[(k * 64 + lane % H) * 2 + 1];
                const float mn = fmaxf(am, om);
                al = al * fast_exp2(am - mn) + ol * fast_exp2(om - mn);
                am = mn;
            }
            m = am;
            l = al;
        }
    }
    static __device__ __forceinline__ float sum(float v, int H, float* lds) {
        for (int off = H; off < (TEAM < 64 ? TEAM : 64); off <<= 1) v += __shfl_xor(v, off);
        if (TEAM > 64) {
            const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
            __syncthreads();
            if (lane < H) lds[w * 64 + lane] = v;
            __syncthreads();
            float acc = 0.f;
            for (int k = 0; k < TEAM / 64; ++k) acc += lds[k * 64 + lane % H];
            v = acc;
        }
        return v;
    }
};

// Both kernels keep a thread's first kSoftmaxHeld values in registers: the loads are issued
// together (one memory latency instead of one per value) and rows of up to kSoftmaxHeld * TEAM
// values — almost all of them — are read once; only longer rows loop and re-read.
constexpr int kSoftmaxHeld = 8;
constexpr int64_t kSoftmaxMaxBlocks = 256 * 32;   // workgroups walk over rows: launching one per few rows costs more than the rows

template <int TEAM>
__global__ void __launch_bounds__(kBlockThreads)
k_edge_softmax(const int64_t* ptr, const int32_t* rows, int64_t row_begin, int64_t row_end, int H,
               float scale2, const float* Z, float* U, float* lse) {
    __shared__ float lds[kBlockThreads * 2];
    constexpr int kTeams = kBlockThreads / TEAM;
    const int t = threadIdx.x % TEAM;
    // a workgroup walks over rows with the grid's stride; the trip count is uniform over the workgroup
    for (int64_t base = row_begin + (int64_t)blockIdx.x * kTeams; base < row_end; base += (int64_t)gridDim.x * kTeams) {
    const int64_t r = base + threadIdx.x / TEAM;
    const bool active = r < row_end;   // uniform over the team (and over the block when TEAM == block)
    int64_t b = 0, e = 0;
    int row = 0;
    if (active) {
        row = rows[r];
        b = ptr[row] * H;
        e = ptr[row + 1] * H;
    }
    float held[kSoftmaxHeld];
    float m = kNegBig, l = 0.f;
#pragma unroll
    for (int k = 0; k < kSoftmaxHeld; ++k) {
        const int64_t x = b + t + (int64_t)k * TEAM;
        held[k] = x < e ? Z[x] * scale2 : -INFINITY;
        m = fmaxf(m, held[k]);
    }
#pragma unroll
    for (int k = 0; k < kSoftmaxHeld; ++k) l += fast_exp2(held[k] - m);   // exp2(-inf) = 0 for the slots past the end
    for (int64_t x = b + t + (int64_t)kSoftmaxHeld * TEAM; x < e; x += TEAM) {
        const float s = Z[x] * scale2;
        const float mn = fmaxf(m, s);
        l = l * fast_exp2(m - mn) + fast_exp2(s - mn);
        m = mn;
    }
    TeamReduce<TEAM>::softmax(m, l, H, lds);
    const float lse2 = m + fast_log2(l);
#pragma unroll
    for (int k = 0; k < kSoftmaxHeld; ++k) {
        const int64_t x = b + t + (int64_t)k * TEAM;
        if (x < e) U[x] = fast_exp2(held[k] - lse2);
    }
    for (int64_t x = b + t + (int64_t)kSoftmaxHeld * TEAM; x < e; x += TEAM) U[x] = fast_exp2(Z[x] * scale2 - lse2);
    if (active && lse && t < H) lse[(int64_t)row * H + t] = e > b ? lse2 * kLn2 : -INFINITY;
    }
}

template <int TEAM>
__global__ void __launch_bounds__(kBlockThreads)
k_edge_softmax_bwd(const int64_t* ptr, const int32_t* rows, int64_t row_begin, int64_t row_end, int H,
                   float scale, const float* U, const float* dU, float* dZ) {
    __shared__ float lds[kBlockThreads * 2];
    constexpr int kTeams = kBlockThreads / TEAM;
    const int t = threadIdx.x % TEAM;
    for (int64_t base = row_begin + (int64_t)blockIdx.x * kTeams; base < row_end; base += (int64_t)gridDim.x * kTeams) {
    const int64_t r = base + threadIdx.x / TEAM;
    int64_t b = 0, e = 0;
    if (r < row_end) {
        const int row = rows[r];
        b = ptr[row] * H;
        e = ptr[row + 1] * H;
    }
    float hu[kSoftmaxHeld], hd[kSoftmaxHeld];
    float dot = 0.f;
#pragma unroll
    for (int k = 0; k < kSoftmaxHeld; ++k) {
        const int64_t x = b + t + (int64_t)k * TEAM;
        hu[k] = x < e ? U[x] : 0.f;
        hd[k] = x < e ? dU[x] : 0.f;
    }
#pragma unroll
    for (int k = 0; k < kSoftmaxHeld; ++k) dot = fmaf(hu[k], hd[k], dot);
    for (int64_t x = b + t + (int64_t)kSoftmaxHeld * TEAM; x < e; x += TEAM) dot = fmaf(U[x], dU[x], dot);
    dot = TeamReduce<TEAM>::sum(dot, H, lds);
#pragma unroll
    for (int k = 0; k < kSoftmaxHeld; ++k) {
        const int64_t x = b + t + (int64_t)k * TEAM;
        if (x < e) dZ[x] = scale * hu[k] * (hd[k] - dot);
    }
    for (int64_t x = b + t + (int64_t)kSoftmaxHeld * TEAM; x < e; x += TEAM) dZ[x] = scale * U[x] * (dU[x] - dot);
    }
}

// The same two kernels with 16 bytes per lane, for H >= 4 (then a row's values start 16-byte
// aligned and a lane's four consecutive values are four consecutive heads: (4 t + c) % H for
// component c, the same for every step since H divides 4 TEAM).  With 4-byte accesses these kernels
// are bound by the number of memory instructions, not by bytes.  Lanes that share heads are H / 4
// apart, so the team reductions run once per component with that stride.
constexpr int kSoftmaxHeld4 = 4;   // float4 per lane held in registers: rows of up to 16 TEAM values are read once

template <int TEAM>
__global__ void __launch_bounds__(kBlockThreads)
k_edge_softmax4(const int64_t* ptr, const int32_t* rows, int64_t row_begin, int64_t row_end, int H,
                float scale2, const float* Z, float* U, float* lse) {
    __shared__ float lds[kBlockThreads * 2];
    constexpr int kTeams = kBlockThreads / TEAM;
    const int t = threadIdx.x % TEAM, HQ = H / 4;
    for (int64_t base = row_begin + (int64_t)blockIdx.x * kTeams; base < row_end; base += (int64_t)gridDim.x * kTeams) {
        const int64_t r = base + threadIdx.x / TEAM;
        const bool active = r < row_end;   // uniform over the team (and over the block when TEAM == block)
        int64_t b = 0, e = 0;
        int row = 0;
        if (active) {
            row = rows[r];
            b = ptr[row] * H;
            e = ptr[row + 1] * H;
        }
        float4 held[kSoftmaxHeld4];
        float m[4] = {kNegBig, kNegBig, kNegBig, kNegBig}, l[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int k = 0; k < kSoftmaxHeld4; ++k) {
            const int64_t x = b + 4 * (t + (int64_t)k * TEAM);
            held[k] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            if (x < e) {
                const float4 z = *reinterpret_cast<const float4*>(Z + x);
                held[k] = make_float4(z.x * scale2, z.y * scale2, z.z * scale2, z.w * scale2);
            }
            m[0] = fmaxf(m[0], held[k].x); m[1] = fmaxf(m[1], held[k].y);
            m[2] = fmaxf(m[2], held[k].z); m[3] = fmaxf(m[3], held[k].w);
        }
#pragma unroll
        for (int k = 0; k < kSoftmaxHeld4; ++k) {   // exp2(-inf) = 0 for the slots past the end
            l[0] += fast_exp2(held[k].x - m[0]); l[1] += fast_exp2(held[k].y - m[1]);
            l[2] += fast_exp2(held[k].z - m[2]); l[3] += fast_exp2(held[k].w - m[3]);
        }
        for (int64_t x = b + 4 * (t + (int64_t)kSoftmaxHeld4 * TEAM); x < e; x += 4 * TEAM) {
            const float4 z = *reinterpret_cast<const float4*>(Z + x);
            const float s[4] = {z.x * scale2, z.y * scale2, z.z * scale2, z.w * scale2};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float mn = fmaxf(m[c], s[c]);
                l[c] = l[c] * fast_exp2(m[c] - mn) + fast_exp2(s[c] - mn);
                m[c] = mn;
            }
        }
        float lse2[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            TeamReduce<TEAM>::softmax(m[c], l[c], HQ, lds);
            lse2[c] = m[c] + fast_log2(l[c]);
        }
#pragma unroll
        for (int k = 0; k < kSoftmaxHeld4; ++k) {
            const int64_t x = b + 4 * (t + (int64_t)k * TEAM);
            if (x < e)
                *reinterpret_cast<float4*>(U + x) =
                    make_float4(fast_exp2(held[k].x - lse2[0]), fast_exp2(held[k].y - lse2[1]),
                                fast_exp2(held[k].z - lse2[2]), fast_exp2(held[k].w - lse2[3]));
        }
        for (int64_t x = b + 4 * (t + (int64_t)kSoftmaxHeld4 * TEAM); x < e; x += 4 * TEAM) {
            const float4 z = *reinterpret_cast<const float4*>(Z + x);
            *reinterpret_cast<float4*>(U + x) =
                make_float4(fast_exp2(z.x * scale2 - lse2[0]), fast_exp2(z.y * scale2 - lse2[1]),
                            fast_exp2(z.z * scale2 - lse2[2]), fast_exp2(z.w * scale2 - lse2[3]));
        }
        if (active && lse && t < HQ) {
            const bool any = e > b;
            *reinterpret_cast<float4*>(lse + (int64_t)row * H + 4 * t) =
                any ? make_float4(lse2[0] * kLn2, lse2[1] * kLn2, lse2[2] * kLn2, lse2[3] * kLn2)
                    : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
        }
    }
}

template <int TEAM>
__global__ void __launch_bounds__(kBlockThreads)
k_edge_softmax_bwd4(const int64_t* ptr, const int32_t* rows, int64_t row_begin, int64_t row_end, int H,
                    float scale, const float* U, const float* dU, float* dZ) {
    __shared__ float lds[kBlockThreads * 2];
    constexpr int kTeams = kBlockThreads / TEAM;
    const int t = threadIdx.x % TEAM, HQ = H / 4;
    for (int64_t base = row_begin + (int64_t)blockIdx.x * kTeams; base < row_end; base += (int64_t)gridDim.x * kTeams) {
        const int64_t r = base + threadIdx.x / TEAM;
        int64_t b = 0, e = 0;
        if (r < row_end) {
            const int row = rows[r];
            b = ptr[row] * H;
            e = ptr[row + 1] * H;
        }
        float4 hu[kSoftmaxHeld4], hd[kSoftmaxHeld4];
        float dot[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int k = 0; k < kSoftmaxHeld4; ++k) {
            const int64_t x = b + 4 * (t + (int64_t)k * TEAM);
            hu[k] = make_float4(0.f, 0.f, 0.f, 0.f);
            hd[k] = hu[k];
            if (x < e) {
                hu[k] = *reinterpret_cast<const float4*>(U + x);
                hd[k] = *reinterpret_cast<const float4*>(dU + x);
            }
        }
#pragma unroll
        for (int k = 0; k < kSoftmaxHeld4; ++k) {
            dot[0] = fmaf(hu[k].x, hd[k].x, dot[0]); dot[1] = fmaf(hu[k].y, hd[k].y, dot[1]);
            dot[2] = fmaf(hu[k].z, hd[k].z, dot[2]); dot[3] = fmaf(hu[k].w, hd[k].w, dot[3]);
        }
        for (int64_t x = b + 4 * (t + (int64_t)kSoftmaxHeld4 * TEAM); x < e; x += 4 * TEAM) {
            const float4 u = *reinterpret_cast<const float4*>(U + x), d = *reinterpret_cast<const float4*>(dU + x);
            dot[0] = fmaf(u.x, d.x, dot[0]); dot[1] = fmaf(u.y, d.y, dot[1]);
            dot[2] = fmaf(u.z, d.z, dot[2]); dot[3] = fmaf(u.w, d.w, dot[3]);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) dot[c] = TeamReduce<TEAM>::sum(dot[c], HQ, lds);
#pragma unroll
        for (int k = 0; k < kSoftmaxHeld4; ++k) {
            const int64_t x = b + 4 * (t + (int64_t)k * TEAM);
            if (x < e)
                *reinterpret_cast<float4*>(dZ + x) =
                    make_float4(scale * hu[k].x * (hd[k].x - dot[0]), scale * hu[k].y * (hd[k].y - dot[1]),
                                scale * hu[k].z * (hd[k].z - dot[2]), scale * hu[k].w * (hd[k].w - dot[3]));
        }
        for (int64_t x = b + 4 * (t + (int64_t)kSoftmaxHeld4 * TEAM); x < e; x += 4 * TEAM) {
            const float4 u = *reinterpret_cast<const float4*>(U + x), d = *reinterpret_cast<const float4*>(dU + x);
            *reinterpret_cast<float4*>(dZ + x) =
                make_float4(scale * u.x * (d.x - dot[0]), scale * u.y * (d.y - dot[1]),
                            scale * u.z * (d.z - dot[2]), scale * u.w * (d.w - dot[3]));
        }
    }
}

template <class T> gta_status run_sddmm(const gta_plan* plan, const Shape& sh, const void* X, const void* Y,
                                        float* Z, float* partial, hipStream_t st) {
#define GTA_CALL(LHc, Gc)                                                                        \
    {                                                                                            \
        using P = SddmmPass<T, LHc, Gc>;                                                         \
        typename P::Params prm{(const char*)X, (const char*)Y, Z, partial, sh.row_bytes, sh.heads}; \
        return launch_pass<P>("sddmm", prm, plan, 0, nullptr, st);                                        \
    }
    GTA_DISPATCH_GEOMETRY(sh.lanes_per_head, sh.lanes_per_row, GTA_CALL)
#undef GTA_CALL
    return GTA_OK;
}

template <class T> gta_status run_spmm(const gta_plan* plan, int side, const Shape& sh, const float* W,
                                       const void* X, void* Y, float* partial, hipStream_t st) {
#define GTA_CALL(LHc, Gc)                                                                        \
    {                                                                                            \
        using P = SpmmPass<T, LHc, Gc>;                                                          \
        typename P::Params prm{W, SegConst{(const char*)X, (const char*)X}, INT32_MAX, (char*)Y, partial, \
                               sh.row_bytes, 1.0f, sh.heads};                                        \
        return launch_pass<P>(side ? "spmm_t" : "spmm", prm, plan, side, side ? plan->t_eid : nullptr, st);                    \
    }
    GTA_DISPATCH_GEOMETRY(sh.lanes_per_head, sh.lanes_per_row, GTA_CALL)
#undef GTA_CALL
    return GTA_OK;
}

bool head_count_ok(int heads) { return heads >= 1 && heads <= 64 && (heads & (heads - 1)) == 0; }

// scratch holds the per-chunk partial results of the row schedules (same sizing as the fused path)
gta_status partial_area(const gta_plan* plan, const Shape& sh, void* scratch, size_t scratch_bytes, float** out) {
    const size_t need = gta_attn_scratch_bytes_min(plan, sh.heads, sh.head_dim, sh.elem_bytes == 4 ? GTA_F32 : GTA_BF16);
    if (!scratch) return fail(GTA_ERR_INVALID_ARG, "scratch is null");
    if (((uintptr_t)scratch & 255) != 0) return fail(GTA_ERR_INVALID_ARG, "scratch must be 256-byte aligned");
    if (scratch_bytes < need) return fail(GTA_ERR_WORKSPACE, "scratch has %zu bytes, %zu needed", scratch_bytes, need);
    *out = static_cast<float*>(scratch);
    return GTA_OK;
}

gta_status check_graph(const gta_plan* plan, const int64_t* indptr, const int32_t* indices, int64_t n_dst,
                       int64_t n_src) {
    if (!plan) return fail(GTA_ERR_INVALID_ARG, "plan is null");
    if (indptr != plan->indptr || (indices && indices != plan->indices))
        return fail(GTA_ERR_INVALID_ARG, "indptr/indices differ from the arrays the plan was built for");
    if (n_dst != plan->n_dst || (n_src >= 0 && n_src != plan->n_src))
        return fail(GTA_ERR_INVALID_ARG, "n_dst/n_src differ from the plan's");
    int device = -1;
    GTA_HIP_TRY(hipGetDevice(&device));
    if (device != plan->device)
        return fail(GTA_ERR_INVALID_ARG, "the plan lives on device %d, the current device is %d", plan->device, device);
    return GTA_OK;
}

}  // namespace
}  // namespace gta

using namespace gta;

extern "C" GTA_API gta_status gta_sddmm(const gta_plan* plan, const int64_t* indptr, const int32_t* indices,
                                        const void* X, const void* Y, float* Z, int64_t n_dst, int64_t n_src,
                                        int heads, int head_dim, gta_dtype dtype, void* scratch,
                                        size_t scratch_bytes, void* stream) {
    gta_status rc = check_graph(plan, indptr, indices, n_dst, n_src);
    if (rc != GTA_OK) return rc;
    Shape sh;
    if ((rc = make_shape(heads, head_dim, dtype, &sh)) != GTA_OK) return rc;
    if ((n_dst > 0 && !X) || (n_src > 0 && !Y) || (plan->nnz > 0 && !Z)) return fail(GTA_ERR_INVALID_ARG, "null tensor pointer");
    if (((uintptr_t)X & 15) || ((uintptr_t)Y & 15)) return fail(GTA_ERR_INVALID_ARG, "tensor base pointers must be 16-byte aligned");
    float* partial;
    if ((rc = partial_area(plan, sh, scratch, scratch_bytes, &partial)) != GTA_OK) return rc;
    if (n_dst == 0) return GTA_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    for (int s = 0; s < sh.n_slices; ++s) {
        const int h0 = s * sh.slice_heads;
        const char* Xs = static_cast<const char*>(X) + (int64_t)h0 * sh.head_bytes;
        const char* Ys = static_cast<const char*>(Y) + (int64_t)h0 * sh.head_bytes;
        rc = sh.elem_bytes == 4 ? run_sddmm<float>(plan, sh, Xs, Ys, Z + h0, partial, st)
                                : run_sddmm<bf16_tag>(plan, sh, Xs, Ys, Z + h0, partial, st);
        if (rc != GTA_OK) return rc;
    }
    return GTA_OK;
}

extern "C" GTA_API gta_status gta_spmm(const gta_plan* plan, const int64_t* indptr, const int32_t* indices,
                                       const float* W, const void* X, void* Y, int64_t n_dst, int64_t n_src,
                                       int heads, int head_dim, gta_dtype dtype, int transposed, void* scratch,
                                       size_t scratch_bytes, void* stream) {
    gta_status rc = check_graph(plan, indptr, indices, n_dst, n_src);
    if (rc != GTA_OK) return rc;
    Shape sh;
    if ((rc = make_shape(heads, head_dim, dtype, &sh)) != GTA_OK) return rc;
    const int64_t rows_out = transposed ? n_src : n_dst, rows_in = transposed ? n_dst : n_src;
    if ((rows_in > 0 && !X) || (rows_out > 0 && !Y) || (plan->nnz > 0 && !W)) return fail(GTA_ERR_INVALID_ARG, "null tensor pointer");
    if (((uintptr_t)X & 15) || ((uintptr_t)Y & 15)) return fail(GTA_ERR_INVALID_ARG, "tensor base pointers must be 16-byte aligned");
    float* partial;
    if ((rc = partial_area(plan, sh, scratch, scratch_bytes, &partial)) != GTA_OK) return rc;
    if (rows_out == 0) return GTA_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int side = transposed ? 1 : 0;
    for (int s = 0; s < sh.n_slices; ++s) {
        const int h0 = s * sh.slice_heads;
        const char* Xs = static_cast<const char*>(X) + (int64_t)h0 * sh.head_bytes;
        char* Ys = static_cast<char*>(Y) + (int64_t)h0 * sh.head_bytes;
        rc = sh.elem_bytes == 4 ? run_spmm<float>(plan, side, sh, W + h0, Xs, Ys, partial, st)
                                : run_spmm<bf16_tag>(plan, side, sh, W + h0, Xs, Ys, partial, st);
        if (rc != GTA_OK) return rc;
    }
    return GTA_OK;
}

namespace {
template <class Launch> gta_status softmax_launches(const gta_plan* plan, int heads, const char* name, Launch launch) {
    const Side& sd = plan->side[0];
    // rows above wave_max_deg: one workgroup each; short rows: 16 lanes each (when the heads fit);
    // the rest: one wavefront each
    if (sd.n_chunked > 0) launch(std::integral_constant<int, kBlockThreads>(), (int64_t)0, sd.n_chunked, sd.n_chunked);
    const Split sp = make_split(plan, 0, 16);
    const int64_t short_begin = heads <= 16 ? sp.pack_begin : sd.n_rows;
    const int64_t mid = short_begin - sd.n_chunked, shorts = sd.n_rows - short_begin;
    if (mid > 0)
        launch(std::integral_constant<int, 64>(), sd.n_chunked, short_begin, (mid + kWavesPerBlock - 1) / kWavesPerBlock);
    if (shorts > 0)
        launch(std::integral_constant<int, 16>(), short_begin, sd.n_rows, (shorts * 16 + kBlockThreads - 1) / kBlockThreads);
    (void)name;
    GTA_HIP_TRY(hipGetLastError());
    return GTA_OK;
}
}  // namespace

extern "C" GTA_API gta_status gta_edge_softmax(const gta_plan* plan, const int64_t* indptr, const float* Z,
                                               float* U, float* lse, int64_t n_dst, int heads, float scale,
                                               void* stream) {
    gta_status rc = check_graph(plan, indptr, nullptr, n_dst, -1);
    if (rc != GTA_OK) return rc;
    if (!head_count_ok(heads)) return fail(GTA_ERR_UNSUPPORTED, "heads must be a power of two <= 64");
    if (!(scale > 0.f)) return fail(GTA_ERR_INVALID_ARG, "scale must be positive");
    if (plan->nnz > 0 && (!Z || !U)) return fail(GTA_ERR_INVALID_ARG, "null tensor pointer");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Side& sd = plan->side[0];
    // 16 bytes per lane when a row's values are 16-byte aligned and a lane's four values are four heads
    const bool vec4 = heads >= 4 && (((uintptr_t)Z | (uintptr_t)U | (uintptr_t)lse) & 15) == 0;
    LaunchTimer t("edge_softmax", sd.n_rows, plan->nnz, st);
    return softmax_launches(plan, heads, "edge_softmax", [&](auto team, int64_t rb, int64_t re, int64_t blocks) {
        const dim3 grid((unsigned)std::min<int64_t>(blocks, kSoftmaxMaxBlocks));
        if (vec4)
            hipLaunchKernelGGL(k_edge_softmax4<decltype(team)::value>, grid, dim3(kBlockThreads), 0, st, sd.ptr,
                               sd.bin_rows, rb, re, heads, scale * kLog2e, Z, U, lse);
        else
            hipLaunchKernelGGL(k_edge_softmax<decltype(team)::value>, grid, dim3(kBlockThreads), 0, st, sd.ptr,
                               sd.bin_rows, rb, re, heads, scale * kLog2e, Z, U, lse);
    });
}

extern "C" GTA_API gta_status gta_edge_softmax_bwd(const gta_plan* plan, const int64_t* indptr, const float* U,
                                                   const float* dU, float* dZ, int64_t n_dst, int heads,
                                                   float scale, void* stream) {
    gta_status rc = check_graph(plan, indptr, nullptr, n_dst, -1);
    if (rc != GTA_OK) return rc;
    if (!head_count_ok(heads)) return fail(GTA_ERR_UNSUPPORTED, "heads must be a power of two <= 64");
    if (!(scale > 0.f)) return fail(GTA_ERR_INVALID_ARG, "scale must be positive");
    if (plan->nnz > 0 && (!U || !dU || !dZ)) return fail(GTA_ERR_INVALID_ARG, "null tensor pointer");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Side& sd = plan->side[0];
    const bool vec4 = heads >= 4 && (((uintptr_t)U | (uintptr_t)dU | (uintptr_t)dZ) & 15) == 0;
    LaunchTimer t("edge_softmax_bwd", sd.n_rows, plan->nnz, st);
    return softmax_launches(plan, heads, "edge_softmax_bwd", [&](auto team, int64_t rb, int64_t re, int64_t blocks) {
        const dim3 grid((unsigned)std::min<int64_t>(blocks, kSoftmaxMaxBlocks));
        if (vec4)
            hipLaunchKernelGGL(k_edge_softmax_bwd4<decltype(team)::value>, grid, dim3(kBlockThreads), 0, st, sd.ptr,
                               sd.bin_rows, rb, re, heads, scale, U, dU, dZ);
        else
            hipLaunchKernelGGL(k_edge_softmax_bwd<decltype(team)::value>, grid, dim3(kBlockThreads), 0, st, sd.ptr,
                               sd.bin_rows, rb, re, heads, scale, U, dU, dZ);
    });
}
