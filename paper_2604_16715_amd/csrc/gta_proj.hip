// Grouped dense projections of the layer on the matrix cores (paper Eq. 3: Q, K, V = X W_Q, X W_K,
// X W_V; Eq. 5: X' = X W_o + Y; and the input gradient dX = dX' W_o^T + dQ W_Q^T + dK W_K^T + dV W_V^T):
//     Y_po[n, d] = sum_{pi < P_IN} X_pi[n, d] * op(W[po][pi]) (+ C_po),      po < P_OUT,
// bf16 operands, fp32 accumulation over ALL P_IN products (rounded once), v_mfma_f32_32x32x16_bf16.
//
// The row operand is what is large (n in the millions, d <= 256), so it is the stationary one: a
// workgroup takes a block of 128 rows, keeps the block's [128 x d] tile of X_pi in LDS and streams
// the weights through LDS in chunks of 32 reduction indices (double-buffered, one workgroup barrier
// per chunk).  Every X_pi is therefore read from HBM exactly once, also when several outputs share
// it (Q, K, V from one read of X), and every Y_po is written once; the weights (<= 128 KB each)
// come out of L2.  The weights are first repacked (k_pack_weights, a few microseconds) so that a
// chunk is one contiguous run in the layout the fragment reads want.
//
// Workgroups are persistent (one per compute unit, walking row blocks with a grid stride): the next
// X tile and the next weight chunk are fetched into registers while the current ones are being
// multiplied, so the global loads of a compute unit never drain.
//
// Fragment convention (lane l of a wavefront, g = l / 32), as in the single-projection kernels:
//   A operand = weight fragment: output column l % 32 of a 32-column tile, 8 consecutive k (8 g ..)
//   B operand = X fragment     : row l % 32 of a 32-row tile, the same 8 k
//   accumulator value v        : row l % 32, column 8 (v / 4) + 4 g + v % 4   (Y transposed: a lane owns
//                                4 consecutive columns of one row per group of four values)
#include "gta_internal.h"

#include <string.h>

namespace gta {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kProjConsumers = 8;                      // multiplying wavefronts of a workgroup
constexpr int kProjThreads = 64 * (kProjConsumers + 4);   // + 2 weight fetchers + 2 X tile fetchers
constexpr int kProjRows = 128, kProjKC = 32, kProjWPitch = kProjKC + 8;
constexpr int kProjMaxParts = 4;

__device__ __forceinline__ bf16x8 frag_of(const u32x4& u) { return __builtin_bit_cast(bf16x8, u); }
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {   // two floats -> two bf16, round to nearest even
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
// LDS exchange between the lanes of ONE wavefront (its LDS instructions execute in order; this only
// keeps the compiler from moving accesses across the exchange)
__device__ __forceinline__ void wave_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---------------------------------------------------------------- weight repacking
// A chunk is the D x 32 slice W_m(k = 32 kc .. 32 kc + 31, all columns), W_m(k, col) being W_m[k * D + col]
// (trans = 0: stored [d_in, d_out]) or W_m[col * D + k] (trans = 1: stored [d_out, d_in]).  Chunks follow each
// other in the order (m, kc); inside a chunk the 16-byte unit u (8 consecutive k of one column) holds
//     column 16 (u / 64) + u % 16,   k = 32 kc + 8 ((u / 16) % 4) .. + 7,
// so 16 consecutive units are the same k piece of 16 consecutive columns.  A fetching wavefront reads
// consecutive units and writes each to its column's LDS row: 16 lanes then write 16 different rows, which at
// the row pitch of 20 dwords fall on different banks (4 lanes per 80-byte row, the plain order, would not).
__device__ __forceinline__ int proj_unit_col(int u) { return 16 * (u >> 6) + (u & 15); }
__device__ __forceinline__ int proj_unit_piece(int u) { return (u >> 4) & 3; }
struct PackArgs { const uint16_t* W[kProjMaxParts * kProjMaxParts]; };
__global__ void __launch_bounds__(256) k_pack_weights(PackArgs a, uint16_t* __restrict__ Wp, int D, int mats, int trans) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t per = (int64_t)D * D;
    if (e >= per * mats) return;
    const int m = (int)(e / per);
    const int r = (int)(e - m * per);
    const int kc = r / (kProjKC * D), in_chunk = r % (kProjKC * D), u = in_chunk / 8;
    const int col = proj_unit_col(u), k = kc * kProjKC + 8 * proj_unit_piece(u) + in_chunk % 8;
    const uint16_t* W = a.W[m];
    Wp[e] = trans ? W[(int64_t)col * D + k] : W[(int64_t)k * D + col];
}

// ---------------------------------------------------------------- the projection kernel
struct ProjArgs {
    const uint16_t* X[kProjMaxParts];   // P_IN inputs  [n, D]
    const uint16_t* C[kProjMaxParts];   // P_OUT addends [n, D] (HAS_C)
    uint16_t* Y[kProjMaxParts];         // P_OUT outputs [n, D]
    const uint16_t* Wp;                 // packed weights, chunk ((po * P_IN + pi) * KCH + kc)
    int64_t n, row_blocks;
};

template <int D> struct ProjShape {
    static constexpr int NTC = D / 32;                      // 32-column tiles of an output
    static constexpr int WAVES_C = D == 64 ? 2 : 4;         // wavefronts across the columns ...
    static constexpr int WAVES_R = 8 / WAVES_C;             // ... and across the 128 rows
    static constexpr int CT = NTC / WAVES_C, RT = 4 / WAVES_R;   // tiles of one wavefront
    static constexpr int XPitch = D + 8;                    // bf16 elements per row of the X tile
    static constexpr int PPitch = 32 * CT + 8;              // ... of a wavefront's result patch
    static constexpr int KCH = D / kProjKC;                 // weight chunks per product
    static constexpr size_t lds_bytes =
        sizeof(uint16_t) * ((size_t)kProjRows * XPitch + 2 * (size_t)D * kProjWPitch + 8 * 32 * (size_t)PPitch);
};

// register sets of a weight-fetching wavefront = weight chunks in flight: four at d = 256 (an L2 round trip
// under load is longer than two chunks' worth of matrix instructions), two for the narrower shapes, whose
// other wavefronts need the registers
constexpr int proj_depth(int kch, bool small_form) { return kch % 8 == 0 && !small_form ? 4 : 2; }

// The walk over (row block, output, input, weight chunk) that every wavefront of a workgroup makes, with
// the workgroup barriers in it; what a wavefront does between the barriers depends on its role (hooks).
template <int P_IN, int P_OUT, int KCH, int DEPTH, class Hooks>
__device__ __forceinline__ void proj_walk(int64_t row_blocks, Hooks& h) {
    constexpr int TOTAL_CHUNKS = P_OUT * P_IN * KCH;
    // Chunk c is multiplied out of LDS buffer c % 2 and travels through register set c % DEPTH of the weight
    // fetchers; both stay compile-time constants because the chunk loop is unrolled DEPTH at a time and a
    // product's chunk count is a multiple of DEPTH.
    static_assert(KCH % DEPTH == 0 && DEPTH % 2 == 0, "chunks per product");
    auto wrap = [](int ci) { return ci % TOTAL_CHUNKS; };   // (TOTAL_CHUNKS can be as small as 2)
    int64_t rb = blockIdx.x;
    if (rb >= row_blocks) return;   // whole workgroup leaves together
    h.prologue(rb);
    __syncthreads();
    int ci = 0;   // chunk being multiplied (even at the top of the pair)
    for (; rb < row_blocks; rb += gridDim.x) {
        // the block after this one (when there is none: this one again, fetched and never used)
        const int64_t next_rb = rb + gridDim.x < row_blocks ? rb + gridDim.x : rb;
#pragma unroll
        for (int po = 0; po < P_OUT; ++po) {
            h.begin_output();
#pragma unroll
            for (int pi = 0; pi < P_IN; ++pi) {
                const bool last_of_block = po == P_OUT - 1 && pi == P_IN - 1;
                // the X tile changes after this product unless the next product reads the same input
                const bool swap_x = P_IN > 1 || po == P_OUT - 1;
                h.begin_product(rb, last_of_block ? next_rb : rb, po, pi, (pi + 1) % P_IN, swap_x);
#pragma unroll 1
                for (int kc = 0; kc < KCH; kc += DEPTH) {
#pragma unroll
                    for (int j = 0; j < DEPTH; ++j) {
                        h.chunk(kc + j, j & 1, (j + 1) % DEPTH, wrap(ci + j + 1 + DEPTH));
                        __syncthreads();
                    }
                    ci = wrap(ci + DEPTH);
                }
                h.end_product(rb, po, pi, swap_x);   // every wavefront has passed the last chunk's barrier: the X tile is free
                if (swap_x) __syncthreads();
            }
        }
    }
}

// 12 wavefronts: 8 multiply (two per SIMD), 2 fetch the weight chunks, 2 fetch the X tiles (one fetcher per
// SIMD).  The multiplying wavefronts issue nothing but fragment reads and matrix instructions between two
// barriers; a fetching wavefront's waits for memory stall nobody else.  Weight and tile fetches are in
// different wavefronts because a wavefront's loads complete in order: behind a tile (HBM latency) every later
// weight chunk (L2 latency) would wait as well.
//
// Row blocks: block rb covers rows [row0, row0 + 128) with row0 = min(128 rb, n - 128), i.e. the last block
// of a tensor whose row count is not a multiple of 128 is moved back so that it is whole (it recomputes
// and rewrites some rows of the block before it with the same bits).  No load or store in the main form
// needs a bounds check that way, which keeps every address "scalar base + one offset register".  Tensors
// of fewer than 128 rows take the SMALL form: one block, rows past the end clamped / not stored.
template <int D, int P_IN, int P_OUT, bool HAS_C, bool SMALL>
__global__ void __launch_bounds__(kProjThreads) __attribute__((amdgpu_waves_per_eu(3, 3)))
k_proj(ProjArgs a) {
    using S = ProjShape<D>;
    constexpr int CT = S::CT, RT = S::RT, XPitch = S::XPitch, PPitch = S::PPitch, KCH = S::KCH;
    constexpr int WPitch = kProjWPitch;
    constexpr int DEPTH = proj_depth(KCH, SMALL);                 // weight chunks in flight
    constexpr int kFetchers = 128;                               // threads of each fetching role
    constexpr int XUnitsPerRow = D / 8, XU = kProjRows * XUnitsPerRow / kFetchers;   // X tile units per fetching thread
    constexpr int WUnits = D * (kProjKC / 8);                    // 16-byte units of a weight chunk
    constexpr int WU = WUnits / kFetchers;
    static_assert(WUnits % kFetchers == 0 && (kProjRows * XUnitsPerRow) % kFetchers == 0, "whole units per fetcher");
    constexpr int UPR = 4 * CT, RPI = 64 / UPR, NI = 32 / RPI;   // result patch: units per row, rows per instruction
    extern __shared__ __align__(16) unsigned char proj_lds[];
    uint16_t* xs = reinterpret_cast<uint16_t*>(proj_lds);        // [128][XPitch]
    uint16_t* ws = xs + kProjRows * XPitch;                      // [2][D][WPitch]
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);      // wavefront index, in a scalar register
    // Global addresses are a per-block base (uniform, kept in scalar registers) plus an unsigned 32-bit byte
    // offset inside the block's 128 x D window.

    if (w < kProjConsumers) {
        // ---------------------------------------------------------------- multiplying wavefronts
        const int g = lane >> 5, r32 = lane & 31;
        const int wr = w / S::WAVES_C, wc = w % S::WAVES_C;
        uint16_t* patch = ws + 2 * D * WPitch + w * (32 * PPitch);   // this wavefront's [32][PPitch]
        const int crow = lane / UPR, cunit = lane % UPR;             // this lane's unit of a patch row group
        const int col0 = wc * CT * 32;                               // first column of this wavefront
        struct Consumer {
            const ProjArgs& a;
            uint16_t *xs, *ws, *patch;
            int g, r32, wr, crow, cunit, col0;
            floatx16 acc[RT][CT];
            u32x4 cregs[HAS_C ? RT * NI : 1];
            __device__ __forceinline__ int64_t row0(int64_t rb) const {   // first row of block rb
                if (SMALL) return 0;
                const int64_t r = rb * kProjRows, last = a.n - kProjRows;
                return r < last ? r : last;
            }
            __device__ __forceinline__ void prologue(int64_t) {}
            __device__ __forceinline__ void begin_output() {
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[rt][ct][v] = 0.f;
            }
            // the addend's tile of this wavefront, in patch-row order, fetched a whole product ahead of its use
            __device__ __forceinline__ void begin_product(int64_t rb, int64_t, int po, int pi, int, bool) {
                if constexpr (HAS_C) {
                    if (pi != P_IN - 1) return;
                    const char* base = reinterpret_cast<const char*>(a.C[po] + row0(rb) * D);
                    const unsigned lim = SMALL ? (unsigned)a.n - 1u : kProjRows - 1u;
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                        for (int q = 0; q < NI; ++q) {
                            unsigned r = (unsigned)((wr * RT + rt) * 32 + RPI * q + crow);
                            if (SMALL) r = r < lim ? r : lim;
                            const unsigned off = (r * D + (unsigned)(col0 + 8 * cunit)) * 2u;
                            cregs[rt * NI + q] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + off));
                        }
                }
            }
            __device__ __forceinline__ void chunk(int kc, int buf, int, int) {   // one weight chunk: two k steps of 16
                const uint16_t* wb = ws + buf * (D * WPitch) + (col0 + r32) * WPitch + 8 * g;
                const uint16_t* xb = xs + (wr * RT * 32 + r32) * XPitch + kc * kProjKC + 8 * g;
                constexpr int KS = kProjKC / 16;
                u32x4 xf[KS][RT], wf[KS][CT];
                // all fragment reads of the chunk first, then the matrix instructions: the reads' latency is paid once
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) xf[ks][rt] = *reinterpret_cast<const u32x4*>(xb + rt * 32 * XPitch + 16 * ks);
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) wf[ks][ct] = *reinterpret_cast<const u32x4*>(wb + ct * 32 * WPitch + 16 * ks);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                        for (int ct = 0; ct < CT; ++ct)
                            acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_of(wf[ks][ct]), frag_of(xf[ks][rt]),
                                                                                  acc[rt][ct], 0, 0, 0);
            }
            // rounds the wavefront's tiles (after adding the addend), lays each 32-row group out row-major in
            // the patch and stores it in whole 16-byte units; rows past the end are not stored
            __device__ __forceinline__ void end_product(int64_t rb, int po, int pi, bool) {
                if (pi != P_IN - 1) return;
                char* ybase = reinterpret_cast<char*>(a.Y[po] + row0(rb) * D);
                const int valid = SMALL ? (int)a.n : kProjRows;
                uint16_t* mine = patch + r32 * PPitch + 4 * g;   // this lane's 8-byte pieces: + 32 ct + 8 (v / 4)
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    if constexpr (HAS_C) {
                        wave_fence();
#pragma unroll
                        for (int q = 0; q < NI; ++q)
                            *reinterpret_cast<u32x4*>(patch + (RPI * q + crow) * PPitch + 8 * cunit) = cregs[rt * NI + q];
                        wave_fence();
#pragma unroll
                        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                            for (int qd = 0; qd < 4; ++qd) {
                                const u32x2 c = *reinterpret_cast<const u32x2*>(mine + 32 * ct + 8 * qd);
                                acc[rt][ct][4 * qd + 0] += __uint_as_float(c.x << 16);
                                acc[rt][ct][4 * qd + 1] += __uint_as_float(c.x & 0xFFFF0000u);
                                acc[rt][ct][4 * qd + 2] += __uint_as_float(c.y << 16);
                                acc[rt][ct][4 * qd + 3] += __uint_as_float(c.y & 0xFFFF0000u);
                            }
                    }
                    wave_fence();
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                        for (int qd = 0; qd < 4; ++qd) {
                            u32x2 o;
                            o.x = pack2(acc[rt][ct][4 * qd + 0], acc[rt][ct][4 * qd + 1]);
                            o.y = pack2(acc[rt][ct][4 * qd + 2], acc[rt][ct][4 * qd + 3]);
                            *reinterpret_cast<u32x2*>(mine + 32 * ct + 8 * qd) = o;
                        }
                    wave_fence();
#pragma unroll
                    for (int q = 0; q < NI; ++q) {
                        const int r = (wr * RT + rt) * 32 + RPI * q + crow;
                        if (!SMALL || r < valid)
                            __builtin_nontemporal_store(
                                *reinterpret_cast<const u32x4*>(patch + (RPI * q + crow) * PPitch + 8 * cunit),
                                reinterpret_cast<u32x4*>(ybase + (unsigned)(r * D + col0 + 8 * cunit) * 2u));
                    }
                }
            }
        } h{a, xs, ws, patch, g, r32, wr, crow, cunit, col0, {}, {}};
        proj_walk<P_IN, P_OUT, KCH, DEPTH>(a.row_blocks, h);
    } else if (w < kProjConsumers + 2) {
        // ---------------------------------------------------------------- weight fetchers
        // While chunk c is multiplied out of LDS buffer c % 2: chunk c + 1 (fetched DEPTH chunks ago) goes from its
        // register set into the other buffer, which was last read before the previous barrier, and chunk
        // c + 1 + DEPTH is fetched into the set that just became free, so an L2 round trip has DEPTH chunks to
        // complete in.
        struct WeightFetcher {
            const ProjArgs& a;
            uint16_t* ws;
            unsigned lt;
            u32x4 regs[DEPTH][WU];
            __device__ __forceinline__ void load(int set, int ci) {
                const char* src = reinterpret_cast<const char*>(a.Wp + (int64_t)ci * (D * kProjKC));
#pragma unroll
                for (int i = 0; i < WU; ++i) regs[set][i] = *reinterpret_cast<const u32x4*>(src + (lt + i * kFetchers) * 16u);
            }
            __device__ __forceinline__ void store(int set, int buf) {
                uint16_t* dst = ws + buf * (D * WPitch);
#pragma unroll
                for (int i = 0; i < WU; ++i) {
                    const int u = (int)lt + i * kFetchers;
                    *reinterpret_cast<u32x4*>(dst + proj_unit_col(u) * WPitch + proj_unit_piece(u) * 8) = regs[set][i];
                }
            }
            __device__ __forceinline__ void prologue(int64_t) {
                constexpr int TOTAL = P_OUT * P_IN * KCH;
                load(0, 0);
                store(0, 0);
#pragma unroll
                for (int t = 1; t < DEPTH; ++t) load(t, t % TOTAL);
                load(0, DEPTH % TOTAL);
            }
            __device__ __forceinline__ void begin_output() {}
            __device__ __forceinline__ void begin_product(int64_t, int64_t, int, int, int, bool) {}
            __device__ __forceinline__ void chunk(int, int buf, int next_set, int fetch_ci) {
                store(next_set, buf ^ 1);
                load(next_set, fetch_ci);
            }
            __device__ __forceinline__ void end_product(int64_t, int, int, bool) {}
        } h{a, ws, (unsigned)tid - 64u * kProjConsumers, {}};
        proj_walk<P_IN, P_OUT, KCH, DEPTH>(a.row_blocks, h);
    } else {
        // ---------------------------------------------------------------- X tile fetchers (one tile ahead)
        struct TileFetcher {
            const ProjArgs& a;
            uint16_t* xs;
            unsigned lt;
            u32x4 regs[XU];
            // thread lt fetches the units (row r0 + i RSTEP, column unit cu): one offset register serves them all,
            // the row step goes into the scalar base
            __device__ __forceinline__ void load(int64_t rb, int pi) {
                constexpr unsigned RSTEP = kFetchers / XUnitsPerRow;
                static_assert(kFetchers % XUnitsPerRow == 0, "a fetching thread stays in one column unit");
                int64_t first = 0;
                if (!SMALL) {
                    const int64_t r = rb * kProjRows, last = a.n - kProjRows;
                    first = r < last ? r : last;
                }
                const char* base = reinterpret_cast<const char*>(a.X[pi] + first * D);
                const unsigned r0 = lt / XUnitsPerRow, cu = lt % XUnitsPerRow;
                if (!SMALL) {
                    const unsigned off = (r0 * D + cu * 8) * 2u;
#pragma unroll
                    for (int i = 0; i < XU; ++i)
                        regs[i] = __builtin_nontemporal_load(
                            reinterpret_cast<const u32x4*>(base + (size_t)i * (RSTEP * D * 2) + off));
                } else {                         // fewer than 128 rows: rows past the end read the last row
                    const unsigned lim = (unsigned)a.n - 1u;
#pragma unroll
                    for (int i = 0; i < XU; ++i) {
                        const unsigned r = r0 + i * RSTEP;
                        regs[i] = __builtin_nontemporal_load(
                            reinterpret_cast<const u32x4*>(base + ((r < lim ? r : lim) * D + cu * 8) * 2u));
                    }
                }
            }
            __device__ __forceinline__ void store() {
                constexpr unsigned RSTEP = kFetchers / XUnitsPerRow;
                uint16_t* dst = xs + (lt / XUnitsPerRow) * XPitch + (lt % XUnitsPerRow) * 8;
#pragma unroll
                for (int i = 0; i < XU; ++i) *reinterpret_cast<u32x4*>(dst + i * (RSTEP * XPitch)) = regs[i];
            }
            __device__ __forceinline__ void prologue(int64_t rb) { load(rb, 0); store(); }
            __device__ __forceinline__ void begin_output() {}
            __device__ __forceinline__ void begin_product(int64_t, int64_t next_tile_rb, int, int, int next_pi, bool swap_x) {
                if (swap_x) load(next_tile_rb, next_pi);
            }
            __device__ __forceinline__ void chunk(int, int, int, int) {}
            __device__ __forceinline__ void end_product(int64_t, int, int, bool swap_x) {
                if (swap_x) store();
            }
        } h{a, xs, (unsigned)tid - 64u * (kProjConsumers + 2), {}};
        proj_walk<P_IN, P_OUT, KCH, DEPTH>(a.row_blocks, h);
    }
}

template <int D, int P_IN, int P_OUT, bool HAS_C, bool SMALL>
gta_status launch_proj_form(const ProjArgs& a, hipStream_t st) {
    constexpr size_t lds = ProjShape<D>::lds_bytes;
    GTA_HIP_TRY(hipFuncSetAttribute((const void*)k_proj<D, P_IN, P_OUT, HAS_C, SMALL>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    int device = 0, cus = 0;
    GTA_HIP_TRY(hipGetDevice(&device));
    GTA_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device));
    if (cus <= 0) cus = 256;
    const int64_t blocks = a.row_blocks < cus ? a.row_blocks : cus;
    hipLaunchKernelGGL((k_proj<D, P_IN, P_OUT, HAS_C, SMALL>), dim3((unsigned)blocks), dim3(kProjThreads), lds, st, a);
    GTA_HIP_TRY(hipGetLastError());
    return GTA_OK;
}
template <int D, int P_IN, int P_OUT, bool HAS_C>
gta_status launch_proj(const ProjArgs& a, hipStream_t st) {
    return a.n < kProjRows ? launch_proj_form<D, P_IN, P_OUT, HAS_C, true>(a, st)
                           : launch_proj_form<D, P_IN, P_OUT, HAS_C, false>(a, st);
}

template <int D> gta_status launch_proj_d(int p_in, int p_out, bool has_c, const ProjArgs& a, hipStream_t st) {
    if (p_in == 1 && p_out == 1) return has_c ? launch_proj<D, 1, 1, true>(a, st) : launch_proj<D, 1, 1, false>(a, st);
    if (p_in == 1 && p_out == 3 && !has_c) return launch_proj<D, 1, 3, false>(a, st);
    if (p_in == 4 && p_out == 1 && !has_c) return launch_proj<D, 4, 1, false>(a, st);
    return fail(GTA_ERR_UNSUPPORTED, "gta_linear_group: supported groupings are 1->1 (with or without addend), "
                                     "1->3 and 4->1 (without)");
}

}  // namespace

bool proj_group_supported(int d, gta_dtype dtype) { return dtype == GTA_BF16 && (d == 64 || d == 128 || d == 256); }
size_t proj_group_scratch_bytes(int d, int mats) { return sizeof(uint16_t) * (size_t)mats * d * d + 256; }

gta_status proj_group(const void* const* X, int p_in, const void* const* W, int p_out, const void* const* C,
                      void* const* Y, int64_t n, int d, int trans_w, void* scratch, size_t scratch_bytes,
                      hipStream_t st) {
    const int mats = p_in * p_out;
    if (p_in < 1 || p_out < 1 || p_in > kProjMaxParts || p_out > kProjMaxParts)
        return fail(GTA_ERR_INVALID_ARG, "between 1 and %d inputs and outputs", kProjMaxParts);
    if (!proj_group_supported(d, GTA_BF16)) return fail(GTA_ERR_UNSUPPORTED, "d must be 64, 128 or 256");
    if (n < 0) return fail(GTA_ERR_INVALID_ARG, "negative size");
    if (!X || !W || !Y) return fail(GTA_ERR_INVALID_ARG, "null pointer argument");
    if (!scratch || ((uintptr_t)scratch & 255) || scratch_bytes < proj_group_scratch_bytes(d, mats))
        return fail(GTA_ERR_WORKSPACE, "scratch must be 256-byte aligned and hold %zu bytes",
                    proj_group_scratch_bytes(d, mats));
    ProjArgs a;
    PackArgs pk;
    memset(&a, 0, sizeof a);
    memset(&pk, 0, sizeof pk);
    bool has_c = false;
    for (int i = 0; i < p_in; ++i) {
        if (n > 0 && (!X[i] || ((uintptr_t)X[i] & 15))) return fail(GTA_ERR_INVALID_ARG, "inputs must be non-null, 16-byte aligned");
        a.X[i] = static_cast<const uint16_t*>(X[i]);
    }
    for (int o = 0; o < p_out; ++o) {
        if (n > 0 && (!Y[o] || ((uintptr_t)Y[o] & 15))) return fail(GTA_ERR_INVALID_ARG, "outputs must be non-null, 16-byte aligned");
        a.Y[o] = static_cast<uint16_t*>(Y[o]);
        a.C[o] = C ? static_cast<const uint16_t*>(C[o]) : nullptr;
        if (a.C[o]) has_c = true;
        if ((uintptr_t)a.C[o] & 15) return fail(GTA_ERR_INVALID_ARG, "addends must be 16-byte aligned");
    }
    if (has_c)
        for (int o = 0; o < p_out; ++o)
            if (!a.C[o]) return fail(GTA_ERR_INVALID_ARG, "either every output has an addend or none has");
    for (int m = 0; m < mats; ++m) {
        if (!W[m] || ((uintptr_t)W[m] & 15)) return fail(GTA_ERR_INVALID_ARG, "weights must be non-null, 16-byte aligned");
        pk.W[m] = static_cast<const uint16_t*>(W[m]);
    }
    if (n == 0) return GTA_OK;
    uint16_t* Wp = static_cast<uint16_t*>(scratch);
    a.Wp = Wp;
    a.n = n;
    a.row_blocks = (n + kProjRows - 1) / kProjRows;
    {
        LaunchTimer t("proj_pack", 0, 0, st);
        const int64_t elems = (int64_t)mats * d * d;
        hipLaunchKernelGGL(k_pack_weights, dim3((unsigned)((elems + 255) / 256)), dim3(256), 0, st, pk, Wp, d, mats,
                           trans_w ? 1 : 0);
    }
    char label[40];
    snprintf(label, sizeof label, "proj_%dto%d%s", p_in, p_out, has_c ? "+C" : "");
    LaunchTimer t(label, n, 0, st);
    switch (d) {
        case 64: return launch_proj_d<64>(p_in, p_out, has_c, a, st);
        case 128: return launch_proj_d<128>(p_in, p_out, has_c, a, st);
        default: return launch_proj_d<256>(p_in, p_out, has_c, a, st);
    }
}

}  // namespace gta

using namespace gta;

extern "C" GTA_API size_t gta_linear_group_scratch_bytes(int d, int p_in, int p_out) {
    if (d <= 0 || p_in < 1 || p_out < 1 || p_in > kProjMaxParts || p_out > kProjMaxParts) return 0;
    return proj_group_scratch_bytes(d, p_in * p_out);
}

extern "C" GTA_API gta_status gta_linear_group(const void* const* X, int p_in, const void* const* W, int p_out,
                                               const void* const* C, void* const* Y, int64_t n, int d,
                                               gta_dtype dtype, int trans_w, void* scratch, size_t scratch_bytes,
                                               void* stream) {
    if (dtype != GTA_BF16) return fail(GTA_ERR_UNSUPPORTED, "gta_linear_group takes bfloat16 tensors");
    return proj_group(X, p_in, W, p_out, C, Y, n, d, trans_w, scratch, scratch_bytes, static_cast<hipStream_t>(stream));
}
