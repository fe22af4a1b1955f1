// Device code shared by the three attention passes (forward, backward by destination row,
// backward by source row).
//
// Data mapping.  One node's row of Q/K/V/... is R = heads*head_dim*sizeof(element) bytes.  A
// *group* of G = R/16 consecutive lanes owns a row: lane l of the group holds bytes
// [16 l, 16 l + 16) — NV = 4 fp32 or 8 bf16 values — so a gather of a neighbour's row is one
// 16-byte load per lane, R contiguous bytes per group.  A head spans LH = head_dim*sizeof/16
// adjacent lanes; per-head dot products are finished with an all-reduce over those LH lanes
// using DPP lane permutes (LH <= 16, always inside one DPP row).
//
// Schedules (picked per degree class by the plan):
//   packed : each group of G lanes takes one row; 64/G rows per wavefront
//   wave   : one row per wavefront; its 64/G groups take alternate entries and are merged
//            with cross-lane shuffles at the end
//   chunk  : one workgroup (4 wavefronts) per chunk of a long row; wavefronts are merged through
//            LDS; a row with several chunks leaves partial results that k_merge combines
// A pass supplies the per-row state, the per-entry gather + arithmetic, the rule that combines
// two partial results, and the final write.
#pragma once
#include "gta_internal.h"

namespace gta {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;   // running-maximum start value (finite: no inf-inf)
constexpr int kBlockThreads = 256;
constexpr int kWavesPerBlock = kBlockThreads / 64;

struct bf16_tag {};

// ---------------------------------------------------------------- element packing
template <class T> struct Elt;
template <> struct Elt<float> {
    static constexpr int NV = 4;
    static __device__ __forceinline__ void unpack(const uint4& r, float (&x)[4]) {
        x[0] = __uint_as_float(r.x); x[1] = __uint_as_float(r.y);
        x[2] = __uint_as_float(r.z); x[3] = __uint_as_float(r.w);
    }
    static __device__ __forceinline__ uint4 pack(const float (&x)[4]) {
        return make_uint4(__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]), __float_as_uint(x[3]));
    }
    // sum of the 4 products of two 16-byte units
    static __device__ __forceinline__ float dot(const uint4& a, const uint4& b) {
        float d = __uint_as_float(a.x) * __uint_as_float(b.x);
        d = fmaf(__uint_as_float(a.y), __uint_as_float(b.y), d);
        d = fmaf(__uint_as_float(a.z), __uint_as_float(b.z), d);
        return fmaf(__uint_as_float(a.w), __uint_as_float(b.w), d);
    }
};
__device__ __forceinline__ uint32_t bf16_round(float x) {   // round to nearest even, upper 16 bits
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;   // NaN
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}
template <> struct Elt<bf16_tag> {
    static constexpr int NV = 8;
    static __device__ __forceinline__ void unpack(const uint4& r, float (&x)[8]) {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            x[2 * k] = __uint_as_float(w[k] << 16);
            x[2 * k + 1] = __uint_as_float(w[k] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ uint4 pack(const float (&x)[8]) {
        uint32_t w[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) w[k] = bf16_round(x[2 * k]) | (bf16_round(x[2 * k + 1]) << 16);
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
    // sum of the 8 products of two 16-byte units, on the packed pairs (v_dot2c_f32_bf16: each
    // product is exact in fp32, accumulation is fp32)
    static __device__ __forceinline__ float dot(const uint4& a, const uint4& b) {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        float d = 0.f;
        d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.x), __builtin_bit_cast(bf16x2, b.x), d, false);
        d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.y), __builtin_bit_cast(bf16x2, b.y), d, false);
        d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.z), __builtin_bit_cast(bf16x2, b.z), d, false);
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.w), __builtin_bit_cast(bf16x2, b.w), d, false);
    }
};

__device__ __forceinline__ uint4 load16(const char* base, int64_t row, int64_t stride, int lig) {
    return *reinterpret_cast<const uint4*>(base + row * stride + lig * 16);
}
// Output rows are written once and not read again by the same pass: non-temporal, so they do not
// push gathered rows out of the caches.
__device__ __forceinline__ void store16(char* base, int64_t row, int64_t stride, int lig, uint4 v) {
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 w = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(base + row * stride + lig * 16));
}
// ... and a row that only its owner reads (never gathered in this pass) is loaded the same way
__device__ __forceinline__ uint4 load16_stream(const char* base, int64_t row, int64_t stride, int lig) {
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + row * stride + lig * 16));
    return make_uint4(w.x, w.y, w.z, w.w);
}
// rows of a two-segment source tensor
__device__ __forceinline__ uint4 load16(const SegConst& t, int split, int row, int64_t stride, int lig) {
    return load16(row < split ? t.lo : t.hi, row, stride, lig);
}
__device__ __forceinline__ void store16(const SegMut& t, int split, int row, int64_t stride, int lig, uint4 v) {
    store16(row < split ? t.lo : t.hi, row, stride, lig, v);
}

// ---------------------------------------------------------------- cross-lane helpers
template <int CTRL> __device__ __forceinline__ float dpp_read(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}
// sum over the LH adjacent lanes of a head; every lane of the head gets the same bits
template <int LH> __device__ __forceinline__ float head_allreduce(float x) {
    static_assert(LH == 1 || LH == 2 || LH == 4 || LH == 8 || LH == 16, "lanes per head");
    if (LH >= 2) x += dpp_read<0xB1>(x);    // quad_perm [1,0,3,2]
    if (LH >= 4) x += dpp_read<0x4E>(x);    // quad_perm [2,3,0,1]
    if (LH >= 8) x += dpp_read<0x141>(x);   // row_half_mirror
    if (LH >= 16) x += dpp_read<0x140>(x);  // row_mirror
    return x;
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// ---------------------------------------------------------------- row sets
struct RowSet {
    const int64_t* ptr;    // row pointer of the pattern being walked
    const int32_t* idx;    // its column ids
    const int32_t* eid;    // walk position -> index into per-entry arrays (null: identity)
    const int32_t* rows;   // plan order of the rows
    const int2* span;      // (ptr[rows[r]], ptr[rows[r] + 1]) per plan position r
    int64_t begin, end;    // this launch covers rows[begin .. end)
};
struct ChunkSet {
    const int64_t* ptr;
    const int32_t* idx;
    const int32_t* eid;
    const int4* chunks;          // (row, begin, end, chunks of row)
    const int32_t* chunk_ptr;    // first chunk of the r-th chunked row
    const int32_t* rows;
    int64_t n_chunks, n_hub;
};

// position of entry `pos` in the caller's per-entry arrays, for passes that read or write them
template <class Pass>
__device__ __forceinline__ int entry_id(const int32_t* eid, int pos, bool valid) {
    if (!Pass::kUsesEntryId || !valid || !eid) return 0;
    return __builtin_nontemporal_load(eid + pos);   // read once
}

// One batch of up to 64 consecutive entries held one per lane (slot t lives in lane lane_base+t).
// The calling group takes slots first, first+stride, ...  The trip count depends only on nb, so
// every lane that shares the batch stays in the loop together: a cross-lane read must never
// name a lane that has already left it.
template <class Pass>
__device__ __forceinline__ void run_batch(Pass& ps, const typename Pass::Params& prm, int my_idx, int my_eid,
                                          bool mapped, int base, int nb, int lane_base, int first, int stride,
                                          int lig) {
    constexpr int U = Pass::U;
    for (int t0 = 0; t0 < nb; t0 += U * stride) {
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u * stride + first;
            ok[u] = t < nb;
            const int j = __shfl(my_idx, (lane_base + t) & 63);
            // entry id of slot t: through the map if there is one, else its position base + t
            const int e = !Pass::kUsesEntryId ? 0 : mapped ? __shfl(my_eid, (lane_base + t) & 63) : base + t;
            ps.load(prm, u, j, e, ok[u], lig);
        }
        ps.compute(ok);
    }
}

// combine the 64/G groups of a wavefront (butterfly over the group index)
template <class Pass> __device__ __forceinline__ void wave_merge(float (&f)[Pass::N]) {
#pragma unroll
    for (int off = Pass::G; off < 64; off <<= 1) {
        float o[Pass::N];
#pragma unroll
        for (int i = 0; i < Pass::N; ++i) o[i] = __shfl_xor(f[i], off);
        Pass::combine(f, o);
    }
}

// ---------------------------------------------------------------- schedules
// Each schedule is a device function of the block index inside its own range, so one launch can
// run all three back to back (longest rows first) or each can be launched by itself.
template <class Pass>
__device__ __forceinline__ void body_packed(const typename Pass::Params& prm, const RowSet& rs, int64_t block) {
    constexpr int G = Pass::G, W = 64 / G;
    const int lane = threadIdx.x & 63, g = lane / G, lig = lane % G;
    const int64_t wave = block * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t r = rs.begin + wave * W + g;
    const bool active = r < rs.end;
    int row = 0, b = 0, e = 0;
    if (active) {   // two independent loads
        row = rs.rows[r];
        const int2 sp = rs.span[r];
        b = sp.x;
        e = sp.y;
    }
    Pass ps;
    ps.init(prm, row, lig, active, true);
    for (int bb = b; bb < e; bb += G) {
        const int nb = min(G, e - bb);
        const int my = lig < nb ? rs.idx[bb + lig] : 0;
        const int my_e = entry_id<Pass>(rs.eid, bb + lig, lig < nb);
        run_batch(ps, prm, my, my_e, rs.eid != nullptr, bb, nb, g * G, 0, 1, lig);
    }
    if (active) Pass::finish(prm, row, lig, ps.f);
}

template <class Pass>
__device__ __forceinline__ void body_wave(const typename Pass::Params& prm, const RowSet& rs, int64_t block) {
    constexpr int G = Pass::G, W = 64 / G;
    const int lane = threadIdx.x & 63, g = lane / G, lig = lane % G;
    const int64_t r = rs.begin + block * kWavesPerBlock + (threadIdx.x >> 6);
    if (r >= rs.end) return;
    const int row = rs.rows[r];
    const int2 sp = rs.span[r];
    const int b = sp.x, e = sp.y;
    Pass ps;
    ps.init(prm, row, lig, true, g == 0);
    for (int bb = b; bb < e; bb += 64) {
        const int nb = min(64, e - bb);
        const int my = lane < nb ? rs.idx[bb + lane] : 0;
        const int my_e = entry_id<Pass>(rs.eid, bb + lane, lane < nb);
        run_batch(ps, prm, my, my_e, rs.eid != nullptr, bb, nb, 0, g, W, lig);
    }
    wave_merge<Pass>(ps.f);
    if (g == 0) Pass::finish(prm, row, lig, ps.f);
}

template <class Pass>
__device__ __forceinline__ void body_chunk(const typename Pass::Params& prm, const ChunkSet& cs, int64_t block,
                                           float (*red)[Pass::N][Pass::G]) {
    constexpr int G = Pass::G, W = 64 / G, N = Pass::N;
    const int lane = threadIdx.x & 63, g = lane / G, lig = lane % G, w = threadIdx.x >> 6;
    const int4 ch = cs.chunks[block];
    const int row = ch.x, cb = ch.y, ce = ch.z;
    const bool first_chunk = (int64_t)cb == cs.ptr[row];
    Pass ps;
    ps.init(prm, row, lig, true, first_chunk && w == 0 && g == 0);
    for (int bb = cb + 64 * w; bb < ce; bb += 64 * kWavesPerBlock) {
        const int nb = min(64, ce - bb);
        const int my = lane < nb ? cs.idx[bb + lane] : 0;
        const int my_e = entry_id<Pass>(cs.eid, bb + lane, lane < nb);
        run_batch(ps, prm, my, my_e, cs.eid != nullptr, bb, nb, 0, g, W, lig);
    }
    wave_merge<Pass>(ps.f);
    if (w > 0 && g == 0) {
#pragma unroll
        for (int i = 0; i < N; ++i) red[w - 1][i][lig] = ps.f[i];
    }
    __syncthreads();
    if (w == 0 && g == 0) {
#pragma unroll
        for (int k = 0; k < kWavesPerBlock - 1; ++k) {
            float o[N];
#pragma unroll
            for (int i = 0; i < N; ++i) o[i] = red[k][i][lig];
            Pass::combine(ps.f, o);
        }
        if (ch.w == 1) {
            Pass::finish(prm, row, lig, ps.f);
        } else {
            float* slot = prm.partial + block * (N * G);
#pragma unroll
            for (int i = 0; i < N; ++i) slot[i * G + lig] = ps.f[i];
        }
    }
}

template <class Pass>
__global__ void __launch_bounds__(kBlockThreads) k_packed(typename Pass::Params prm, RowSet rs) {
    body_packed<Pass>(prm, rs, blockIdx.x);
}
template <class Pass>
__global__ void __launch_bounds__(kBlockThreads) k_wave(typename Pass::Params prm, RowSet rs) {
    body_wave<Pass>(prm, rs, blockIdx.x);
}
template <class Pass>
__global__ void __launch_bounds__(kBlockThreads) k_chunk(typename Pass::Params prm, ChunkSet cs) {
    __shared__ float red[kWavesPerBlock - 1][Pass::N][Pass::G];
    body_chunk<Pass>(prm, cs, blockIdx.x, red);
}

// all three schedules in one grid: blocks [0, n_chunks) run chunks, the next wave_blocks run
// one row per wavefront, the rest run packed rows
struct FusedRanges { int64_t wave_blocks; RowSet wave, packed; };
template <class Pass>
__global__ void __launch_bounds__(kBlockThreads) k_rows(typename Pass::Params prm, ChunkSet cs, FusedRanges fr) {
    __shared__ float red[kWavesPerBlock - 1][Pass::N][Pass::G];
    const int64_t b = blockIdx.x;
    if (b < cs.n_chunks) body_chunk<Pass>(prm, cs, b, red);
    else if (b < cs.n_chunks + fr.wave_blocks) body_wave<Pass>(prm, fr.wave, b - cs.n_chunks);
    else body_packed<Pass>(prm, fr.packed, b - cs.n_chunks - fr.wave_blocks);
}

// rows that were cut into several chunks: combine their partial results in chunk order
template <class Pass>
__global__ void __launch_bounds__(kBlockThreads) k_merge(typename Pass::Params prm, ChunkSet cs) {
    constexpr int G = Pass::G, W = 64 / G, N = Pass::N;
    const int lane = threadIdx.x & 63, g = lane / G, lig = lane % G;
    const int64_t r = ((int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6)) * W + g;
    if (r >= cs.n_hub) return;
    const int row = cs.rows[r];
    const int c0 = cs.chunk_ptr[r], c1 = cs.chunk_ptr[r + 1];
    float f[N];
    const float* slot = prm.partial + (int64_t)c0 * (N * G);
#pragma unroll
    for (int i = 0; i < N; ++i) f[i] = slot[i * G + lig];
    for (int c = c0 + 1; c < c1; ++c) {
        slot = prm.partial + (int64_t)c * (N * G);
        float o[N];
#pragma unroll
        for (int i = 0; i < N; ++i) o[i] = slot[i * G + lig];
        Pass::combine(f, o);
    }
    Pass::finish(prm, row, lig, f);
}

// ---------------------------------------------------------------- launching a pass
// One launch covers every row of the side (plus the small merge launch when hub rows exist).
// entry_map translates a position in the walked pattern into an index of the caller's per-entry
// arrays (null: the position itself); only passes with kUsesEntryId look at it.
// With split timing requested each schedule gets its own launch so it can be timed by itself.
template <class Pass>
gta_status launch_pass(const char* name, const typename Pass::Params& prm, const gta_plan* plan, int side,
                       const int32_t* entry_map, hipStream_t st) {
    constexpr int W = 64 / Pass::G;
    const Side& sd = plan->side[side];
    const Split sp = make_split(plan, side, Pass::G);
    char label[40];
    ChunkSet cs{sd.ptr, sd.idx, entry_map, sd.chunks, sd.chunk_ptr, sd.bin_rows, sd.n_chunks, sd.n_hub};
    const RowSet wave{sd.ptr, sd.idx, entry_map, sd.bin_rows, sd.span, sp.wave_begin, sp.wave_end};
    const RowSet packed{sd.ptr, sd.idx, entry_map, sd.bin_rows, sd.span, sp.pack_begin, sp.pack_end};
    const int64_t wave_blocks = (sp.wave_end - sp.wave_begin + kWavesPerBlock - 1) / kWavesPerBlock;
    const int64_t per_block = kWavesPerBlock * W;
    const int64_t pack_blocks = (sp.pack_end - sp.pack_begin + per_block - 1) / per_block;
    const int64_t merge_blocks = (sd.n_hub + per_block - 1) / per_block;
    auto merge = [&]() {
        if (sd.n_hub <= 0) return;
        snprintf(label, sizeof label, "%s.merge", name);
        LaunchTimer t(label, sd.n_hub, 0, st);
        hipLaunchKernelGGL(k_merge<Pass>, dim3((unsigned)merge_blocks), dim3(kBlockThreads), 0, st, prm, cs);
    };
    if (!split_launches()) {
        const int64_t blocks = sd.n_chunks + wave_blocks + pack_blocks;
        if (blocks > 0) {
            LaunchTimer t(name, sd.n_rows, sp.chunk_entries + sp.wave_entries + sp.pack_entries, st);
            hipLaunchKernelGGL(k_rows<Pass>, dim3((unsigned)blocks), dim3(kBlockThreads), 0, st, prm, cs,
                               FusedRanges{wave_blocks, wave, packed});
        }
        merge();
    } else {
        if (sd.n_chunks > 0) {
            snprintf(label, sizeof label, "%s.chunk", name);
            LaunchTimer t(label, sd.n_chunked, sp.chunk_entries, st);
            hipLaunchKernelGGL(k_chunk<Pass>, dim3((unsigned)sd.n_chunks), dim3(kBlockThreads), 0, st, prm, cs);
        }
        merge();
        if (wave_blocks > 0) {
            snprintf(label, sizeof label, "%s.wave", name);
            LaunchTimer t(label, sp.wave_end - sp.wave_begin, sp.wave_entries, st);
            hipLaunchKernelGGL(k_wave<Pass>, dim3((unsigned)wave_blocks), dim3(kBlockThreads), 0, st, prm, wave);
        }
        if (pack_blocks > 0) {
            snprintf(label, sizeof label, "%s.packed", name);
            LaunchTimer t(label, sp.pack_end - sp.pack_begin, sp.pack_entries, st);
            hipLaunchKernelGGL(k_packed<Pass>, dim3((unsigned)pack_blocks), dim3(kBlockThreads), 0, st, prm, packed);
        }
    }
    GTA_HIP_TRY(hipGetLastError());
    return GTA_OK;
}

// Expands to a switch over the supported (lanes per head, lanes per row) pairs.
#define GTA_DISPATCH_GEOMETRY(LHv, Gv, CALL)                                                   \
    switch ((LHv) * 100 + (Gv)) {                                                              \
        case 104: CALL(1, 4); break;   case 108: CALL(1, 8); break;                            \
        case 116: CALL(1, 16); break;  case 132: CALL(1, 32); break;                           \
        case 164: CALL(1, 64); break;  case 204: CALL(2, 4); break;                            \
        case 404: CALL(4, 4); break;                                                           \
        case 208: CALL(2, 8); break;   case 216: CALL(2, 16); break;                           \
        case 232: CALL(2, 32); break;  case 264: CALL(2, 64); break;                           \
        case 408: CALL(4, 8); break;   case 416: CALL(4, 16); break;                           \
        case 432: CALL(4, 32); break;  case 464: CALL(4, 64); break;                           \
        case 808: CALL(8, 8); break;   case 816: CALL(8, 16); break;                           \
        case 832: CALL(8, 32); break;  case 864: CALL(8, 64); break;                           \
        case 1616: CALL(16, 16); break; case 1632: CALL(16, 32); break;                        \
        case 1664: CALL(16, 64); break;                                                        \
        default: return fail(GTA_ERR_UNSUPPORTED, "unsupported row geometry");                 \
    }

template <int G> struct UnrollFor { static constexpr int value = G == 64 ? 8 : 4; };

}  // namespace gta
