// Dense projections of the layer (paper Eq. 3: Q,K,V = X W_Q, X W_K, X W_V; Eq. 5: X' = X W_o + Y)
// and their gradients, on the matrix cores: bf16 operands, fp32 accumulation,
// v_mfma_f32_32x32x16_bf16.  These are the only dense contractions of the layer; problem sizes
// are n x d x d with n in the millions and d <= 512 (Section 4.1), so one operand is a tall
// matrix streamed once from HBM and the other a small weight that lives in LDS.
//
// Fragment convention used throughout (lane l of a wavefront, g = l / 32):
//   A operand: row l % 32, the 8 consecutive k values 8 g .. 8 g + 7 of the current 16-wide k step
//   B operand: column l % 32, the same 8 k values
//   C/D      : 16 floats; value v belongs to row 8 (v / 4) + 4 g + v % 4, column l % 32
// A and B only have to agree with each other on which k values a lane holds.
#include "gta_internal.h"

namespace gta {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kTile = 128;       // output tile edge of a workgroup
constexpr int kPad = 8;          // bf16 elements of padding per LDS row (16 bytes)

__device__ __forceinline__ bf16x8 as_frag(const uint4& u) { return __builtin_bit_cast(bf16x8, u); }
__device__ __forceinline__ int out_row(int v, int lane) { return 8 * (v / 4) + 4 * (lane / 32) + v % 4; }
__device__ __forceinline__ uint32_t bf16_bits(float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ float bf16_value(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
// 16-bit element e (0..7) of a 16-byte unit
__device__ __forceinline__ uint32_t half_of(const uint4& u, int e) {
    const uint32_t wd = (e >> 1) == 0 ? u.x : (e >> 1) == 1 ? u.y : (e >> 1) == 2 ? u.z : u.w;
    return (wd >> ((e & 1) * 16)) & 0xFFFFu;
}

// ---------------------------------------------------------------------------------------------
// Y[n, d_out] = X[n, d_in] * op(W) (+ C).  A workgroup owns one column tile of op(W) (COLS = 64 or
// 128 columns, template argument NT = COLS / 32), staged in LDS once ("k contiguous"); after that
// its WAVES (4 or 8) wavefronts never synchronise with each other.  Wavefront w walks over 32-row
// tiles of X (rows 32 w .. 32 w + 31 of the workgroup's 32 WAVES-row tiles).  The weight fragment is the MFMA's A operand and the X fragment its B operand, so the
// accumulator holds Y transposed: a lane owns ONE row of Y (l % 32) and, per group of four
// accumulator values, four consecutive columns — 8 bytes of the row once rounded to bf16.  The
// 32 x COLS result goes through a per-wavefront LDS patch in 8-byte pieces and leaves in coalesced
// 16-byte stores; an addend C comes in the same way.
//   W_KMAJOR = true : W is stored [d_out, d_in] (Y = X W^T)   -> panel rows are copied
//   W_KMAJOR = false: W is stored [d_in, d_out] (Y = X W)     -> panel is transposed while staged
// Workgroups whose ids differ by 8 (same XCD) take the same row tiles for different column tiles,
// so the rows of X they all read come out of one L2.
constexpr int kStepsPerChunk = 8;                   // k steps (of 16) staged per chunk
constexpr int kStagePitch = 16 * kStepsPerChunk + kPad;   // bf16 elements per row of a wavefront's 32-row X stage
// (the result patch, 32 rows of up to 128 columns plus padding, reuses the stage)

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

inline size_t linear_lds_bytes(int d_in, int cols, int waves) {
    return sizeof(uint16_t) * ((size_t)cols * (d_in + kPad) + (size_t)(32 * waves) * kStagePitch);
}

// LDS traffic between the lanes of ONE wavefront: the hardware executes a wavefront's LDS
// instructions in order; this only stops the compiler from moving accesses across the exchange.
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// two floats -> two bf16 (round to nearest even) in one dword: v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Fast form (KSTEPS = d_in / 16 at compile time for d_in = 64, 128, 256; d_out a multiple of 64):
// the main loop has no data-dependent branch at all.  Every load and store is unconditional —
// rows past the end are clamped to the last row, whose values they then recompute and store once
// more — so the compiler can count the memory operations in flight exactly and wait only for the
// ones it needs; any guarded access inside the loop makes it wait for all of them, which ends the
// run-ahead.  The generic form (KSTEPS = 0) takes any d_in, d_out with bounds checks and no run-ahead.
template <bool W_KMAJOR, int KSTEPS, bool HAS_C, int NT, int WAVES>
__global__ void __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_linear(const uint16_t* __restrict__ X, const uint16_t* __restrict__ W, const uint16_t* __restrict__ C,
         uint16_t* __restrict__ Y, int64_t n, int d_in_arg, int d_out, int col_tiles, int64_t row_tiles,
         int64_t groups_per_xcd) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    constexpr int COLS = 32 * NT;                    // columns of Y per workgroup
    constexpr int THREADS = 64 * WAVES, ROWS = 32 * WAVES;   // ... and rows of one of its row tiles
    constexpr int kPatchPitch = COLS + kPad;         // bf16 elements per row of the result patch
    constexpr int UPR = COLS / 8, RPI = 64 / UPR, NI = 32 / RPI;   // result tile: 16-byte units per row, rows per
                                                                   // instruction, instructions per 32-row tile
    static_assert(kPatchPitch <= kStagePitch, "the patch lives in the stage");
    const int d_in = KSTEPS > 0 ? KSTEPS * 16 : d_in_arg;
    const int pitch = d_in + kPad;
    uint16_t* panel = reinterpret_cast<uint16_t*>(lds_raw);                 // [64][d_in + kPad]
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 5, r32 = lane & 31;
    uint16_t* stage = panel + COLS * pitch + (32 * w) * kStagePitch;   // this wavefront's [32][kStagePitch]
    uint16_t* patch = stage;                                                    // the result patch reuses it
    const int64_t b = blockIdx.x, j = b >> 3;
    const int xcd = (int)(b & 7);
    const int col0 = (int)(j % col_tiles) * COLS;
    const int64_t group = j / col_tiles;   // 0 .. groups_per_xcd-1; row tiles (group + m * groups_per_xcd) * 8 + xcd

    if (W_KMAJOR) {   // 16-byte units of the panel's rows, zero beyond d_out
        const int units_per_k = d_in / 8;
        for (int u = threadIdx.x; u < COLS * units_per_k; u += THREADS) {
            const int c = u / units_per_k, ku = u - c * units_per_k;
            uint4 val = make_uint4(0, 0, 0, 0);
            if (col0 + c < d_out) val = *reinterpret_cast<const uint4*>(W + (int64_t)(col0 + c) * d_in + ku * 8);
            *reinterpret_cast<uint4*>(panel + c * pitch + ku * 8) = val;
        }
    } else {          // two k rows x 8 columns per step; consecutive lanes take consecutive k pairs
        const int pairs = d_in / 2;
        for (int u = threadIdx.x; u < pairs * (COLS / 8); u += THREADS) {
            const int cu = u / pairs, kp = u - cu * pairs;
            uint4 v0 = make_uint4(0, 0, 0, 0), v1 = v0;
            if (col0 + cu * 8 < d_out) {
                v0 = *reinterpret_cast<const uint4*>(W + (int64_t)(2 * kp) * d_out + col0 + cu * 8);
                v1 = *reinterpret_cast<const uint4*>(W + (int64_t)(2 * kp + 1) * d_out + col0 + cu * 8);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e)
                *reinterpret_cast<uint32_t*>(panel + (cu * 8 + e) * pitch + 2 * kp) = half_of(v0, e) | (half_of(v1, e) << 16);
        }
    }
    __syncthreads();   // the only workgroup-wide synchronisation: the panel is complete

    // 32-row tiles of this wavefront: rows 32 w .. of the 128-row tiles (group + m * groups_per_xcd) * 8 + xcd
    const int64_t first_tile = group * 8 + xcd, tile_stride = groups_per_xcd * 8;
    auto tile_row0 = [&](int64_t m) { return (first_tile + m * tile_stride) * ROWS + 32 * w; };
    int64_t my_tiles = first_tile < row_tiles ? (row_tiles - first_tile + tile_stride - 1) / tile_stride : 0;
    // A wavefront whose 32 rows of the last row block all lie past the end skips that tile: with
    // clamped rows it would recompute row n - 1 and, when Y aliases C, could read an addend that
    // the row's owner has already updated.  (Rows past the end INSIDE a tile are harmless: their
    // addend loads and stores go with the owner's, in the same instructions' order.)
    if (my_tiles > 0 && tile_row0(my_tiles - 1) >= n) --my_tiles;
    if (my_tiles == 0) return;
    floatx16 acc[NT];   // acc[t][v]: row r32, column 32 t + 8 (v / 4) + 4 g + v % 4 of the wavefront's 32 x COLS tile
    uint16_t* my_patch = patch + r32 * kPatchPitch + 4 * g;   // this lane's 8-byte pieces: + 32 t + 8 (v / 4)

    auto add_patch = [&]() {   // acc += the bf16 tile that was just written to the patch (row-major)
        wave_lds_fence();
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const u32x2 c = *reinterpret_cast<const u32x2*>(my_patch + 32 * t + 8 * qd);
                acc[t][4 * qd + 0] += __uint_as_float(c.x << 16);
                acc[t][4 * qd + 1] += __uint_as_float(c.x & 0xFFFF0000u);
                acc[t][4 * qd + 2] += __uint_as_float(c.y << 16);
                acc[t][4 * qd + 3] += __uint_as_float(c.y & 0xFFFF0000u);
            }
    };
    auto acc_to_patch = [&]() {   // round and lay the tile out row-major in the patch
        wave_lds_fence();         // earlier reads of the patch / stage by this wavefront are issued
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                u32x2 o;
                o.x = pack_bf16x2(acc[t][4 * qd + 0], acc[t][4 * qd + 1]);
                o.y = pack_bf16x2(acc[t][4 * qd + 2], acc[t][4 * qd + 3]);
                *reinterpret_cast<u32x2*>(my_patch + 32 * t + 8 * qd) = o;
            }
        wave_lds_fence();
    };

    if constexpr (KSTEPS > 0) {
        // X goes global -> registers -> this wavefront's LDS stage -> MFMA fragments, in chunks of
        // up to 8 k steps (256 bytes per row).  The global loads are fully coalesced (a load
        // instruction covers 4 rows x 256 contiguous bytes = 8 whole cache lines; reading the
        // fragments directly would touch 32 lines per instruction and is bound by the L1's line
        // rate) and run two chunks — one tile at d_in = 256 — ahead in two register sets.  The
        // addend's 32 x 64 tile travels with the chunk that completes its tile.
        constexpr int CS = KSTEPS < kStepsPerChunk ? KSTEPS : kStepsPerChunk;   // k steps per chunk
        constexpr int CHUNKS = KSTEPS / CS;              // 1 or 2; even steps are chunk 0 when 2
        constexpr int UNITS = CS * 2;                    // 16-byte units per row of a chunk
        constexpr int ROWS_PER_LOAD = 64 / UNITS;        // rows one load instruction covers
        constexpr int LOADS = 32 / ROWS_PER_LOAD;        // load instructions per chunk
        static_assert(CHUNKS == 1 || CHUNKS == 2, "a tile is one or two chunks");
        const int64_t steps = my_tiles * CHUNKS;         // step s = (tile s / CHUNKS, chunk s % CHUNKS)
        const int urow = lane / UNITS, ucol = lane % UNITS;
        const int crow = lane / UPR, cunit = lane % UPR, ccol = col0 + 8 * cunit;   // addend / result units
        const int64_t last_row = n - 1;
        u32x4 set0[LOADS], set1[LOADS];   // the X units of the even / odd steps (then of the step two later)
        u32x4 cset0[NI], cset1[NI];       // the addend tiles that belong to them
#define GTA_FETCH_X(SET, STEP, ODD)                                                                \
        {                                                                                          \
            int64_t fs = (STEP);                                                                   \
            if (fs >= steps) fs = steps - 1; /* past the end: re-read the last tile (unused) */    \
            const int64_t frow0 = tile_row0(fs / CHUNKS);                                          \
            constexpr int fk = (CHUNKS == 1 ? 0 : (ODD)) * (16 * CS);                              \
            _Pragma("unroll") for (int q = 0; q < LOADS; ++q) {                                    \
                int64_t row = frow0 + q * ROWS_PER_LOAD + urow;                                    \
                row = row < last_row ? row : last_row;                                             \
                SET[q] = *reinterpret_cast<const u32x4*>(X + row * d_in + fk + 8 * ucol);          \
            }                                                                                      \
        }
#define GTA_FETCH_C(CSET, STEP, ODD)                                                               \
        if constexpr (HAS_C && (CHUNKS == 1 || (ODD))) {                                           \
            int64_t fs = (STEP);                                                                   \
            if (fs >= steps) fs = steps - 1;                                                       \
            const int64_t frow0 = tile_row0(fs / CHUNKS);                                          \
            _Pragma("unroll") for (int q = 0; q < NI; ++q) {                                       \
                int64_t row = frow0 + RPI * q + crow;                                              \
                row = row < last_row ? row : last_row;                                             \
                CSET[q] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(C + row * d_out + ccol)); \
            }                                                                                      \
        }
#define GTA_STEP(SET, CSET, STEP, ODD, AHEAD)                                                      \
        {                                                                                          \
            const int64_t s = (STEP);                                                              \
            constexpr int chunk = CHUNKS == 1 ? 0 : (ODD);                                         \
            wave_lds_fence(); /* earlier fragment / patch reads of this wavefront are issued */    \
            _Pragma("unroll") for (int q = 0; q < LOADS; ++q)                                      \
                *reinterpret_cast<u32x4*>(stage + (q * ROWS_PER_LOAD + urow) * kStagePitch + 8 * ucol) = SET[q]; \
            if (AHEAD) GTA_FETCH_X(SET, s + 2, ODD)                                                \
            __builtin_amdgcn_sched_barrier(0);                                                     \
            wave_lds_fence();                                                                      \
            if (chunk == 0) {                                                                      \
                _Pragma("unroll") for (int t = 0; t < NT; ++t)                                     \
                    _Pragma("unroll") for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;                \
            }                                                                                      \
            const uint16_t* wrow = panel + r32 * pitch + chunk * (16 * CS) + 8 * g;                \
            const uint16_t* xrow = stage + r32 * kStagePitch + 8 * g;                              \
            _Pragma("unroll") for (int i = 0; i < CS; ++i) {                                       \
                const uint4 xf = *reinterpret_cast<const uint4*>(xrow + 16 * i);                   \
                _Pragma("unroll") for (int t = 0; t < NT; ++t) {                                   \
                    const uint4 wf = *reinterpret_cast<const uint4*>(wrow + 32 * t * pitch + 16 * i); \
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(wf), as_frag(xf), acc[t], 0, 0, 0); \
                }                                                                                  \
            }                                                                                      \
            if (chunk == CHUNKS - 1) {                                                             \
                const int64_t row0 = tile_row0(s / CHUNKS);                                        \
                if constexpr (HAS_C) {                                                             \
                    wave_lds_fence();                                                              \
                    _Pragma("unroll") for (int q = 0; q < NI; ++q)                                 \
                        *reinterpret_cast<u32x4*>(patch + (RPI * q + crow) * kPatchPitch + 8 * cunit) = CSET[q]; \
                    add_patch();                                                                   \
                }                                                                                  \
                acc_to_patch();                                                                    \
                _Pragma("unroll") for (int q = 0; q < NI; ++q) {                                   \
                    int64_t row = row0 + RPI * q + crow;                                           \
                    row = row < last_row ? row : last_row;                                         \
                    __builtin_nontemporal_store(                                                   \
                        *reinterpret_cast<const u32x4*>(patch + (RPI * q + crow) * kPatchPitch + 8 * cunit), \
                        reinterpret_cast<u32x4*>(Y + row * d_out + ccol));                         \
                }                                                                                  \
                if (AHEAD) GTA_FETCH_C(CSET, s + 2, ODD)                                           \
            }                                                                                      \
        }
        GTA_FETCH_X(set0, 0, 0)
        GTA_FETCH_C(cset0, 0, 0)
        GTA_FETCH_X(set1, 1, 1)
        GTA_FETCH_C(cset1, 1, 1)
        int64_t s0 = 0;
        for (; s0 + 1 < steps; s0 += 2) {
            GTA_STEP(set0, cset0, s0, 0, true)
            GTA_STEP(set1, cset1, s0 + 1, 1, true)
        }
        if (s0 < steps) GTA_STEP(set0, cset0, s0, 0, false)   // an odd number of one-chunk tiles
#undef GTA_STEP
#undef GTA_FETCH_C
#undef GTA_FETCH_X
    } else {
        // any shape: fragments are fetched when needed (no run-ahead), every access is bounds-checked
        const int ksteps = d_in / 16;
        for (int64_t m = 0; m < my_tiles; ++m) {
            const int64_t row0 = tile_row0(m);
            int64_t row = row0 + r32;
            if (row >= n) row = n - 1;   // computed, never stored
            const uint16_t* src = X + row * d_in + 8 * g;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
            for (int i = 0; i < ksteps; ++i) {
                const uint4 xf = *reinterpret_cast<const uint4*>(src + 16 * i);
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const uint4 wf = *reinterpret_cast<const uint4*>(panel + (32 * t + r32) * pitch + 16 * i + 8 * g);
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(wf), as_frag(xf), acc[t], 0, 0, 0);
                }
            }
            if (C) {
                wave_lds_fence();   // the patch may still be read by this wavefront's previous stores
#pragma unroll
                for (int q = 0; q < NI; ++q) {   // 32 rows x UPR units of 8 columns
                    const int u = lane + 64 * q, r = u / UPR, cu = u % UPR;
                    uint4 c = make_uint4(0, 0, 0, 0);
                    if (row0 + r < n && col0 + cu * 8 < d_out)
                        c = *reinterpret_cast<const uint4*>(C + (row0 + r) * d_out + col0 + cu * 8);
                    *reinterpret_cast<uint4*>(patch + r * kPatchPitch + cu * 8) = c;
                }
                add_patch();
            }
            acc_to_patch();
#pragma unroll
            for (int q = 0; q < NI; ++q) {
                const int u = lane + 64 * q, r = u / UPR, cu = u % UPR;
                if (row0 + r < n && col0 + cu * 8 < d_out)
                    *reinterpret_cast<uint4*>(Y + (row0 + r) * d_out + col0 + cu * 8) =
                        *reinterpret_cast<const uint4*>(patch + r * kPatchPitch + cu * 8);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// dW[d_in, d_out] = X^T dY, summed over the n rows.  A workgroup of WI x WO wavefronts owns a
// TI x TO tile of dW (TI = 32 WI AI, TO = 32 WO AO) over one block of rows; wavefront (wi, wo) owns
// AI x AO accumulator tiles of 32 x 32.  Two shapes are used: 128 x 128 with 4 wavefronts, and
// 256 x 256 with 8 wavefronts when a dimension exceeds 128 — there a workgroup covers the whole
// gradient at d = 256, so X and dY are each read exactly once (a gradient that fits ONE such tile
// takes k_linear_dw_direct further down instead; this kernel serves the other shapes).  Both operands have the reduction
// index (the row) as their slow index, so each 32-row block is transposed into LDS: a thread loads
// 4 consecutive rows of the same 8 columns and writes one 8-byte word per column.  LDS rows are 18
// dwords apart and consecutive lanes write consecutive row quads, which spreads both the 8-byte
// writes and the 8-byte fragment reads over all banks.  The LDS block is double-buffered (one
// workgroup barrier per 32 rows; the next block is written while the current one is multiplied) and
// the global loads run Q blocks ahead in registers.
// Row blocks are reduced afterwards in a fixed order (k_reduce_partials): no atomics.
constexpr int kDwKB = 32, kDwPitch = kDwKB + 4;   // rows per block; 36 bf16 = 18 dwords per LDS row

template <int WI, int WO, int AI, int AO>
constexpr size_t dw_lds_bytes() { return sizeof(uint16_t) * 2 * (size_t)(32 * WI * AI + 32 * WO * AO) * kDwPitch; }

// A launch covers up to four products.  The workgroups of one row split that belong to different
// products get consecutive places on the same XCD, so they run side by side: where two products name
// the same X, the rows one of them brings into that XCD's L2 serve the other (KEEP_X: X is then read
// with ordinary loads; an operand nobody else reads stays non-temporal).
struct DwOperands { const uint16_t* X[4]; const uint16_t* dY[4]; };
struct DwResults { float* dW[4]; };

template <int WI, int WO, int AI, int AO, int Q, bool KEEP_X>
__global__ void __launch_bounds__(64 * WI * WO, 8 / (WI * WO))   // 8 wavefronts per compute unit
k_linear_dw(DwOperands ops, int products, float* __restrict__ partial,
            int64_t n, int d_in, int d_out, int64_t rows_per_split, int tiles_i, int tiles_o, int splits) {
    constexpr int T = 64 * WI * WO, TI = 32 * WI * AI, TO = 32 * WO * AO, KB = kDwKB, pitch = kDwPitch;
    static_assert(TI == T / 2 && TO == T / 2, "half of the threads stage X, the other half dY, one unit each");
    static_assert(Q % 2 == 0, "the buffer a queue slot goes to must not depend on the outer iteration");
    static_assert(KB == 32, "a row block is two MFMA steps of 16 rows");
    extern __shared__ __align__(16) unsigned char dw_lds[];
    uint16_t* xs = reinterpret_cast<uint16_t*>(dw_lds);   // [2][TI][pitch]
    uint16_t* ys = xs + 2 * TI * pitch;                   // [2][TO][pitch]
    const int lane = threadIdx.x & 63, g = lane >> 5, r32 = lane & 31;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wavefront index, in a scalar register
    // the products and tiles of one row split get ids 8 apart (same XCD) so that the rows they share
    // hit in one L2
    const int64_t bid = blockIdx.x, jj = bid >> 3;
    const int tiles = tiles_i * tiles_o;
    const int product = (int)(jj % products);
    const int tile = (int)((jj / products) % tiles);
    const int64_t split = (jj / products / tiles) * 8 + (bid & 7);
    if (split >= splits) return;   // whole workgroup leaves together
    const uint16_t* X = product == 0 ? ops.X[0] : product == 1 ? ops.X[1] : product == 2 ? ops.X[2] : ops.X[3];
    const uint16_t* dY = product == 0 ? ops.dY[0] : product == 1 ? ops.dY[1] : product == 2 ? ops.dY[2] : ops.dY[3];
    const int i0 = (tile % tiles_i) * TI, o0 = (tile / tiles_i) * TO;
    const int64_t rbeg = split * rows_per_split;   // < n: the host rounds splits so that none is empty
    const int64_t rend = rbeg + rows_per_split < n ? rbeg + rows_per_split : n;
    const int wi = w / WO, wo = w % WO;

    // Loader role, per wavefront: the first half of the wavefronts stage X, the others dY; a thread's
    // unit is 8 columns x 4 rows.  The operand's base and row length sit in scalar registers and the
    // thread's place inside a row block is one 32-bit byte offset that never changes, so a load in
    // the loop costs no vector arithmetic.  A unit past the last column (a ragged tile) reads
    // column 0 instead: it only feeds gradient entries that are never stored.
    const bool loads_x = w < WI * WO / 2;
    const int lt = threadIdx.x % (T / 2), rq = lt & 7, cu = lt >> 3;
    const uint16_t* src = loads_x ? X : dY;
    const int ld = loads_x ? d_in : d_out;
    int cbase = (loads_x ? i0 : o0) + cu * 8;
    if (cbase >= ld) cbase = 0;
    const unsigned row_bytes = 2u * (unsigned)ld;
    const unsigned voff = (unsigned)(rq * 4) * row_bytes + 2u * (unsigned)cbase;
    uint16_t* dst = (loads_x ? xs : ys) + (cu * 8) * pitch + rq * 4;
    constexpr int buf_stride = T / 2 * pitch;   // elements between the two buffers of an operand

    floatx16 acc[AI][AO];
#pragma unroll
    for (int a = 0; a < AI; ++a)
#pragma unroll
        for (int b = 0; b < AO; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // register queue: a slot holds the unit of one row block; its loads are issued Q + 1 blocks ahead
    uint4 queue[Q][4];
    auto load16 = [&](const char* p) {   // an operand read once is non-temporal (wavefront-uniform choice)
        const u32x4* q = reinterpret_cast<const u32x4*>(p);
        const u32x4 v = KEEP_X && loads_x ? *q : __builtin_nontemporal_load(q);
        return make_uint4(v.x, v.y, v.z, v.w);
    };
    auto fetch_whole = [&](uint4 (&slot)[4], int64_t r0) {   // a block that lies inside the split: no checks
        const char* base = reinterpret_cast<const char*>(src + r0 * ld);
#pragma unroll
        for (int q = 0; q < 4; ++q) slot[q] = load16(base + (size_t)q * row_bytes + voff);
    };
    auto fetch = [&](uint4 (&slot)[4], int64_t r0) {         // any block: rows past the end count as zero
        if (r0 + KB <= rend) {
            fetch_whole(slot, r0);
        } else if (r0 < rend) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int64_t r = r0 + rq * 4 + q;
                const uint4 v = load16(reinterpret_cast<const char*>(src + (r < rend ? r : rbeg) * ld + cbase));
                slot[q] = r < rend ? v : make_uint4(0, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) slot[q] = make_uint4(0, 0, 0, 0);
        }
    };
    // unit of four rows of one operand -> LDS: each column of the unit becomes one 8-byte word (byte
    // permutes pick the low or the high halves of two rows' dwords)
    auto stage = [&](const uint4 (&slot)[4], int buf) {
        uint16_t* my_dst = dst + buf * buf_stride;
        const uint32_t* s0 = reinterpret_cast<const uint32_t*>(&slot[0]);
        const uint32_t* s1 = reinterpret_cast<const uint32_t*>(&slot[1]);
        const uint32_t* s2 = reinterpret_cast<const uint32_t*>(&slot[2]);
        const uint32_t* s3 = reinterpret_cast<const uint32_t*>(&slot[3]);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            constexpr uint32_t LOW = 0x05040100u, HIGH = 0x07060302u;
            *reinterpret_cast<uint2*>(my_dst + (2 * c) * pitch) =
                make_uint2(__builtin_amdgcn_perm(s1[c], s0[c], LOW), __builtin_amdgcn_perm(s3[c], s2[c], LOW));
            *reinterpret_cast<uint2*>(my_dst + (2 * c + 1) * pitch) =
                make_uint2(__builtin_amdgcn_perm(s1[c], s0[c], HIGH), __builtin_amdgcn_perm(s3[c], s2[c], HIGH));
        }
    };
    // MFMA operands of one 16-row step, two register sets (one is multiplied while the other is read)
    uint4 fa[2][AI], fb[2][AO];
    auto fragments = [&](int set, int buf, int ks) {   // rows are 8-byte aligned only: two 8-byte reads each
        const uint16_t* xb = xs + buf * buf_stride + (32 * AI * wi + r32) * pitch + 8 * g + ks;
        const uint16_t* yb = ys + buf * buf_stride + (32 * AO * wo + r32) * pitch + 8 * g + ks;
#pragma unroll
        for (int t = 0; t < AI; ++t) {
            const uint2* pa = reinterpret_cast<const uint2*>(xb + 32 * t * pitch);
            const uint2 a0 = pa[0], a1 = pa[1];
            fa[set][t] = make_uint4(a0.x, a0.y, a1.x, a1.y);
        }
#pragma unroll
        for (int t = 0; t < AO; ++t) {
            const uint2* pb = reinterpret_cast<const uint2*>(yb + 32 * t * pitch);
            const uint2 b0 = pb[0], b1 = pb[1];
            fb[set][t] = make_uint4(b0.x, b0.y, b1.x, b1.y);
        }
    };
    auto multiply = [&](int set) {
#pragma unroll
        for (int a = 0; a < AI; ++a)
#pragma unroll
            for (int b = 0; b < AO; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(fa[set][a]), as_frag(fb[set][b]), acc[a][b], 0, 0, 0);
    };

    // Block b lives in LDS buffer b & 1 and came through queue slot b % Q (Q is even, so inside the
    // unrolled loop both are functions of i alone).  A block is multiplied in two halves, and each
    // half hides the memory work of the next one:
    //   first half  (rows 0-15 of block b, operands read earlier)  | reads the operands of rows 16-31
    //                                                              | and writes block b + 1 to the other buffer
    //   barrier
    //   second half (rows 16-31)                                   | reads the operands of rows 0-15 of
    //                                                              | block b + 1, issues the loads of block b + 1 + Q
    // The other buffer was last read for block b - 1, and those reads were complete when the wavefront
    // reached the previous barrier; what is written before a barrier is read after it.  Blocks past
    // the end of the split hold zeros.
#pragma unroll
    for (int i = 0; i < Q; ++i) fetch(queue[i], rbeg + (int64_t)i * KB);
    stage(queue[0], 0);
    fetch(queue[0], rbeg + (int64_t)Q * KB);
    __syncthreads();
    fragments(0, 0, 0);
    // The main loop runs while every block it fetches is a whole one and has no branch inside, so the
    // wait for a queue slot leaves the newer slots' loads in flight; the last blocks take the checked form.
    int64_t rb = rbeg;
    for (; rb + (int64_t)(2 * Q + 1) * KB <= rend; rb += (int64_t)Q * KB) {
#pragma unroll
        for (int i = 0; i < Q; ++i) {
            fragments(1, i & 1, 16);
            stage(queue[(i + 1) % Q], (i + 1) & 1);
            multiply(0);
            __syncthreads();
            fragments(0, (i + 1) & 1, 0);
            fetch_whole(queue[(i + 1) % Q], rb + (int64_t)(i + Q + 1) * KB);
            multiply(1);
        }
    }
    for (; rb < rend; rb += (int64_t)Q * KB) {
#pragma unroll
        for (int i = 0; i < Q; ++i) {
            const int64_t r0 = rb + (int64_t)i * KB;
            if (r0 >= rend) break;   // uniform over the workgroup
            fragments(1, i & 1, 16);
            stage(queue[(i + 1) % Q], (i + 1) & 1);
            multiply(0);
            __syncthreads();
            fragments(0, (i + 1) & 1, 0);
            fetch(queue[(i + 1) % Q], r0 + (int64_t)(Q + 1) * KB);
            multiply(1);
        }
    }
    float* out = partial + ((int64_t)product * splits + split) * d_in * d_out;
#pragma unroll
    for (int a = 0; a < AI; ++a)
#pragma unroll
        for (int b = 0; b < AO; ++b) {
            const int o = o0 + 32 * AO * wo + 32 * b + r32;
            if (o >= d_out) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = i0 + 32 * AI * wi + 32 * a + out_row(v, lane);
                if (i < d_in) out[(int64_t)i * d_out + o] = acc[a][b][v];
            }
        }
}

// ---------------------------------------------------------------------------------------------
// The 256 x 256 tile of X^T dY again, with the memory path of this chip: global memory goes straight
// into LDS (global_load_lds, 16 bytes per lane, no registers in between), four row blocks are resident
// so that three are in flight while one is multiplied, and the MFMA operands come out of LDS through
// transposing reads (ds_read_b64_tr_b16), which turn the row-major blocks into "8 consecutive rows of
// one column" per lane.  Nothing but matrix, LDS and load instructions is left in the loop, and the
// accumulation order is that of k_linear_dw (same row splits, same 16-row steps): same bits.
//
// LDS image of one operand's 32-row x 256-column block (16 KB), in 16-byte units (one row, 8 columns):
//   unit (k, c) with k the row and c = column / 8 sits at ((k / 4) * 8 + c / 4) * 16 + (k % 4) * 4 + c % 4,
// i.e. 4 rows x 32 columns make one 256-byte group.  A load instruction fills 1 KB = 4 groups = 4 rows x
// 128 columns: lane u fetches row 4 (k / 4) + (u % 16) / 4, unit 4 (group) + u % 4 (256 contiguous bytes
// per row).  A transposing read returns to lane j of every 16 lanes element j % 4 of the 8-byte pieces
// that lanes j / 4, j / 4 + 4, j / 4 + 8, j / 4 + 12 point at; with those four pointing at the same four
// columns in rows k .. k + 3 the lane gets four consecutive rows of one column, and the 32 lanes of half
// a wavefront touch exactly one 256-byte group: no bank conflicts.
constexpr int kDdBufs = 4;
constexpr int kDdPanelBytes = kDwKB * 256 * 2;                          // 16 KB
constexpr size_t kDdLdsBytes = (size_t)kDdBufs * 2 * kDdPanelBytes;     // 128 KB
__device__ __align__(16) unsigned int g_dd_zero_unit[4];                // what rows past the end read

typedef short short4v __attribute__((ext_vector_type(4)));
#define GTA_LDS_PTR(T, p) reinterpret_cast<__attribute__((address_space(3))) T*>(reinterpret_cast<uintptr_t>(p))

template <bool KEEP_X>
__global__ void __launch_bounds__(512, 1)
k_linear_dw_direct(DwOperands ops, int products, float* __restrict__ partial, int64_t n, int d_in, int d_out,
                   int64_t rows_per_split, int splits) {
    constexpr int KB = kDwKB, AI = 4, AO = 2, WO = 4;
    extern __shared__ __align__(16) unsigned char dd_lds[];   // [buffer][X panel | dY panel]
    const int lane = threadIdx.x & 63, g = lane >> 5, r32 = lane & 31;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t bid = blockIdx.x, jj = bid >> 3;
    const int product = (int)(jj % products);
    const int64_t split = (jj / products) * 8 + (bid & 7);
    if (split >= splits) return;   // whole workgroup leaves together
    const uint16_t* X = product == 0 ? ops.X[0] : product == 1 ? ops.X[1] : product == 2 ? ops.X[2] : ops.X[3];
    const uint16_t* dY = product == 0 ? ops.dY[0] : product == 1 ? ops.dY[1] : product == 2 ? ops.dY[2] : ops.dY[3];
    const int64_t rbeg = split * rows_per_split;   // < n: the host rounds splits so that none is empty
    const int64_t rend = rbeg + rows_per_split < n ? rbeg + rows_per_split : n;
    const int wi = w / WO, wo = w % WO;

    // loader role: wavefronts 0-3 bring X, 4-7 dY; wavefront wq of an operand fills KB 4 wq .. 4 wq + 3 of
    // the block's 16 (instruction q = 0..3: rows 8 wq + 4 (q / 2) .. + 3, columns 128 (q % 2) .. + 127)
    const bool loads_x = w < 4;
    const int wq = w & 3;
    const uint16_t* src = loads_x ? X : dY;
    const int ld = loads_x ? d_in : d_out;
    const unsigned row_bytes = 2u * (unsigned)ld;
    const int krow = lane % 16 / 4;                     // row of the lane inside the 4-row group
    unsigned voff[2];                                    // byte offset of the lane's unit, for q % 2 = 0, 1
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        int c = 4 * (4 * h + lane / 16) + lane % 4;      // column unit
        if (c * 8 >= ld) c = 0;                          // past the last column: feeds entries never stored
        voff[h] = (unsigned)(8 * wq + krow) * row_bytes + 16u * (unsigned)c;
    }
    // The loads are written as assembly on purpose: the compiler then knows nothing of memory instructions
    // that write LDS, and leaves their completion (vmcnt) to the waits placed by hand below; it would
    // otherwise wait for ALL of them before any LDS read it cannot prove independent.  m0 holds the LDS
    // byte address of the instruction's 1 KB; lane l's 16 bytes land at m0 + 16 l.
    const bool keep = KEEP_X && loads_x;   // an operand read once is non-temporal (wavefront-uniform choice)
    const unsigned my_panel = (unsigned)reinterpret_cast<uintptr_t>(GTA_LDS_PTR(unsigned char, dd_lds)) +
                              (loads_x ? 0u : (unsigned)kDdPanelBytes) + (unsigned)wq * 4096u;
    auto issue_whole = [&](int buf, int64_t r0) {   // a block that lies inside the split: no checks
        const char* base0 = reinterpret_cast<const char*>(src + r0 * ld);
        const char* base1 = base0 + 4 * (size_t)row_bytes;
        const unsigned dst = my_panel + (unsigned)buf * (2u * kDdPanelBytes);
#define GTA_DD_ISSUE(CACHE)                                                                                 \
        asm volatile("s_mov_b32 m0, %4\n\ts_nop 0\n\t"                                                       \
                     "global_load_lds_dwordx4 %0, %2" CACHE "\n\t"                                           \
                     "s_add_u32 m0, m0, 0x400\n\ts_nop 0\n\t"                                               \
                     "global_load_lds_dwordx4 %1, %2" CACHE "\n\t"                                           \
                     "s_add_u32 m0, m0, 0x400\n\ts_nop 0\n\t"                                               \
                     "global_load_lds_dwordx4 %0, %3" CACHE "\n\t"                                           \
                     "s_add_u32 m0, m0, 0x400\n\ts_nop 0\n\t"                                               \
                     "global_load_lds_dwordx4 %1, %3" CACHE                                                  \
                     : : "v"(voff[0]), "v"(voff[1]), "s"(base0), "s"(base1), "s"(dst) : "memory", "scc", "m0")
        if (keep) GTA_DD_ISSUE(""); else GTA_DD_ISSUE(" nt");
#undef GTA_DD_ISSUE
    };
    auto issue = [&](int buf, int64_t r0) {         // the last block: rows past the end read zeros
        const unsigned dst = my_panel + (unsigned)buf * (2u * kDdPanelBytes);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int64_t r = r0 + 8 * wq + 4 * (q / 2) + krow;
            const char* p = reinterpret_cast<const char*>(src + r0 * ld) + (size_t)(q / 2) * 4 * row_bytes + voff[q % 2];
            if (r >= rend) p = reinterpret_cast<const char*>(g_dd_zero_unit);
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                         : : "v"(p), "s"(dst + (unsigned)q * 1024u) : "memory", "m0");
        }
    };

    // operand fragments: lane l supplies the address of row (l % 16) / 4 of its 16-lane group's four rows
    // and of the 8-byte piece l % 4 of the group's 16 columns; the rows of a group are 8 g + 4 r .. + 3
    const unsigned lane_off = (unsigned)(g * 4096 + ((lane % 16 / 4) * 4 + 2 * (lane / 16 % 2) + lane % 4 / 2) * 16 + (lane & 1) * 8);
    const unsigned char* xfrag = dd_lds + lane_off + (AI * wi) * 256;
    const unsigned char* yfrag = dd_lds + kDdPanelBytes + lane_off + (AO * wo) * 256;
    uint4 fa[2][AI], fb[2][AO];
    auto tr8 = [&](const unsigned char* p) {   // 8 consecutive rows of the lane's column: two transposing reads
        const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(GTA_LDS_PTR(short4v, p));
        const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(GTA_LDS_PTR(short4v, p + 2048));
        const uint2 a = __builtin_bit_cast(uint2, lo), b = __builtin_bit_cast(uint2, hi);
        return make_uint4(a.x, a.y, b.x, b.y);
    };
    auto fragments = [&](int set, int buf, int ks) {
        const int o = buf * (2 * kDdPanelBytes) + (ks / 4) * 2048;
#pragma unroll
        for (int t = 0; t < AI; ++t) fa[set][t] = tr8(xfrag + o + t * 256);
#pragma unroll
        for (int t = 0; t < AO; ++t) fb[set][t] = tr8(yfrag + o + t * 256);
    };
    floatx16 acc[AI][AO];
#pragma unroll
    for (int a = 0; a < AI; ++a)
#pragma unroll
        for (int b = 0; b < AO; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    auto multiply = [&](int set) {
#pragma unroll
        for (int a = 0; a < AI; ++a)
#pragma unroll
            for (int b = 0; b < AO; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(fa[set][a]), as_frag(fb[set][b]), acc[a][b], 0, 0, 0);
    };

    // Block b lives in buffer b % 4.  While block b is multiplied, blocks b + 1 .. b + 3 are on their way
    // (b + 3 is requested first thing; its buffer held block b - 1, whose last reads were complete at the
    // previous barrier).  A wavefront's loads complete in order, so "at most 8 outstanding" means that its
    // part of block b + 1 has landed; the barrier then makes every wavefront's part visible.  The first
    // half of a block is multiplied while the second half's operands are read, the second half while the
    // first operands of the next block are read.
    const int64_t nwhole = (rend - rbeg) / KB, nblocks = (rend - rbeg + KB - 1) / KB;
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        if (j < nwhole) issue_whole(j, rbeg + (int64_t)j * KB);
        else if (j < nblocks) issue(j, rbeg + (int64_t)j * KB);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    fragments(0, 0, 0);
    int64_t b = 0;
    for (; b + 6 < nwhole; b += 4) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            issue_whole((i + 3) % 4, rbeg + (b + i + 3) * KB);
            fragments(1, i, 16);
            multiply(0);
            asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
            __syncthreads();
            fragments(0, (i + 1) % 4, 0);
            multiply(1);
        }
    }
    for (; b < nblocks; b += 4) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (b + i >= nblocks) break;   // uniform over the workgroup
            if (b + i + 3 < nwhole) issue_whole((i + 3) % 4, rbeg + (b + i + 3) * KB);
            else if (b + i + 3 < nblocks) issue((i + 3) % 4, rbeg + (b + i + 3) * KB);
            fragments(1, i, 16);
            multiply(0);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            fragments(0, (i + 1) % 4, 0);   // past the last block: stale data, never multiplied
            multiply(1);
        }
    }
    float* out = partial + ((int64_t)product * splits + split) * d_in * d_out;
#pragma unroll
    for (int a = 0; a < AI; ++a)
#pragma unroll
        for (int bb = 0; bb < AO; ++bb) {
            const int o = 32 * AO * wo + 32 * bb + r32;
            if (o >= d_out) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = 32 * AI * wi + 32 * a + out_row(v, lane);
                if (i < d_in) out[(int64_t)i * d_out + o] = acc[a][bb][v];
            }
        }
}

// Sums the row splits' partial results in a fixed order: a workgroup takes 32 consecutive elements of
// product blockIdx.y; thread (element e, group j of 8) adds splits j, j + 8, ... and the 8 group sums
// are then added in group order.
__global__ void __launch_bounds__(256)
k_reduce_partials(const float* __restrict__ partials, DwResults res, int64_t elems, int splits) {
    __shared__ float part[8][32];
    const int e = threadIdx.x & 31, j = threadIdx.x >> 5, product = blockIdx.y;
    const int64_t i = (int64_t)blockIdx.x * 32 + e;
    const float* partial = partials + (int64_t)product * splits * elems;
    float* dW = product == 0 ? res.dW[0] : product == 1 ? res.dW[1] : product == 2 ? res.dW[2] : res.dW[3];
    float acc = 0.f;
    if (i < elems)
        for (int s = j; s < splits; s += 8) acc += partial[(int64_t)s * elems + i];
    part[j][e] = acc;
    __syncthreads();
    if (j == 0 && i < elems) {
        float total = part[0][e];
#pragma unroll
        for (int k = 1; k < 8; ++k) total += part[k][e];
        dW[i] = total;
    }
}

struct DwGeometry { int tile, tiles_i, tiles_o, splits; int64_t rows_per_split; };

// tile: 256 when a dimension exceeds 128 (bf16 only: the 256 x 256 shape), else 128
DwGeometry dw_geometry(int64_t n, int d_in, int d_out, gta_dtype dtype) {
    DwGeometry g;
    g.tile = dtype == GTA_BF16 && (d_in > kTile || d_out > kTile) ? 256 : kTile;
    g.tiles_i = (d_in + g.tile - 1) / g.tile;
    g.tiles_o = (d_out + g.tile - 1) / g.tile;
    const int64_t tiles = (int64_t)g.tiles_i * g.tiles_o;
    int64_t splits = (g.tile == 256 ? 256 : 512) / tiles;   // 8 wavefronts per compute unit (the register budget) in total
    const int64_t max_splits = (n + 511) / 512;         // at least 512 rows per split
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    g.rows_per_split = ((n + splits - 1) / splits + 31) / 32 * 32;
    if (g.rows_per_split < 32) g.rows_per_split = 32;
    g.splits = (int)((n + g.rows_per_split - 1) / g.rows_per_split);
    if (g.splits < 1) g.splits = 1;
    return g;
}

gta_status check_dims(int d_in, int d_out, gta_dtype dtype) {
    if (dtype != GTA_BF16 && dtype != GTA_F32) return fail(GTA_ERR_UNSUPPORTED, "unknown dtype %d", (int)dtype);
    if (d_in <= 0 || d_out <= 0 || d_in % 16 != 0 || d_out % 8 != 0)
        return fail(GTA_ERR_UNSUPPORTED, "d_in must be a multiple of 16 and d_out a multiple of 8");
    if (d_in > 4096 || d_out > 4096) return fail(GTA_ERR_UNSUPPORTED, "dimensions up to 4096 are supported");
    return GTA_OK;
}

}  // namespace
}  // namespace gta

using namespace gta;

extern "C" GTA_API gta_status gta_linear(const void* X, const void* W, const void* C, void* Y, int64_t n,
                                         int d_in, int d_out, gta_dtype dtype, int trans_w, void* stream) {
    gta_status rc = check_dims(d_in, d_out, dtype);
    if (rc != GTA_OK) return rc;
    if (d_in > 512) return fail(GTA_ERR_UNSUPPORTED, "d_in <= 512 is supported (the weight panel must fit in LDS)");
    if (n < 0) return fail(GTA_ERR_INVALID_ARG, "negative size");
    if (n == 0) return GTA_OK;
    if (!X || !W || !Y) return fail(GTA_ERR_INVALID_ARG, "null tensor pointer");
    if (((uintptr_t)X & 15) || ((uintptr_t)W & 15)) return fail(GTA_ERR_INVALID_ARG, "X and W must be 16-byte aligned");
    if (((uintptr_t)Y & 15) || ((uintptr_t)C & 15)) return fail(GTA_ERR_INVALID_ARG, "Y and C must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == GTA_F32)
        return launch_linear_f32((const float*)X, (const float*)W, (const float*)C, (float*)Y, n, d_in, d_out,
                                 trans_w, st);
    // Shape of a workgroup.  Every column tile of a row block re-reads the block's rows of X (out of
    // L2), so wider column tiles mean less traffic; the weight panel of the tile has to fit in LDS
    // next to the wavefronts' stages, with 8 wavefronts per compute unit in all (the register budget):
    //   d_in <= 128, d_out % 128 == 0: 128 columns, 4 wavefronts, two workgroups per compute unit
    //   d_in == 256, d_out % 128 == 0: 128 columns, 8 wavefronts, one workgroup per compute unit
    //   otherwise                     : 64 columns, 4 wavefronts, two per compute unit
    // The branch-free form needs whole column tiles and a compile-time d_in.
    const bool known_k = d_in == 64 || d_in == 128 || d_in == 256;
    const bool wide = d_out % 128 == 0 && known_k;
    const int cols = wide ? 128 : 64;
    const int waves = wide && d_in == 256 ? 8 : 4;
    const bool fast = d_out % cols == 0 && known_k;
    const size_t lds = linear_lds_bytes(d_in, cols, waves);
    const int col_tiles = (d_out + cols - 1) / cols;
    const int64_t row_tiles = (n + 32 * waves - 1) / (32 * waves);
    // 8 wavefronts per compute unit in total
    int64_t groups_per_xcd = (waves == 8 ? 32 : 64) / col_tiles;
    if (groups_per_xcd < 1) groups_per_xcd = 1;
    const int64_t max_groups = (row_tiles + 7) / 8;
    if (groups_per_xcd > max_groups) groups_per_xcd = max_groups;
    const int64_t blocks = groups_per_xcd * col_tiles * 8;
    LaunchTimer t(trans_w ? "linear_nt" : "linear_nn", n, 0, st);
#define GTA_LAUNCH_LINEAR(KM, KS, HC, NT, WV)                                                                      \
    do {                                                                                                           \
        GTA_HIP_TRY(hipFuncSetAttribute((const void*)k_linear<KM, KS, HC, NT, WV>,                                 \
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                    \
        hipLaunchKernelGGL((k_linear<KM, KS, HC, NT, WV>), dim3((unsigned)blocks), dim3(64 * WV), lds, st,         \
                           (const uint16_t*)X, (const uint16_t*)W, (const uint16_t*)C, (uint16_t*)Y, n, d_in,      \
                           d_out, col_tiles, row_tiles, groups_per_xcd);                                           \
    } while (0)
#define GTA_LINEAR_BY_C(KM, KS, NT, WV)                      \
    if (C) GTA_LAUNCH_LINEAR(KM, KS, true, NT, WV); else GTA_LAUNCH_LINEAR(KM, KS, false, NT, WV)
#define GTA_LINEAR_BY_K(KM)                                                                                  \
    switch (fast ? d_in : 0) {                                                                               \
        case 64: if (wide) { GTA_LINEAR_BY_C(KM, 4, 4, 4); } else { GTA_LINEAR_BY_C(KM, 4, 2, 4); } break;   \
        case 128: if (wide) { GTA_LINEAR_BY_C(KM, 8, 4, 4); } else { GTA_LINEAR_BY_C(KM, 8, 2, 4); } break;  \
        case 256: if (wide) { GTA_LINEAR_BY_C(KM, 16, 4, 8); } else { GTA_LINEAR_BY_C(KM, 16, 2, 4); } break; \
        default: GTA_LAUNCH_LINEAR(KM, 0, false, 2, 4); break;                                               \
    }
    if (trans_w) { GTA_LINEAR_BY_K(true) } else { GTA_LINEAR_BY_K(false) }
#undef GTA_LINEAR_BY_K
#undef GTA_LINEAR_BY_C
#undef GTA_LAUNCH_LINEAR
    GTA_HIP_TRY(hipGetLastError());
    return GTA_OK;
}

extern "C" GTA_API size_t gta_linear_dw_scratch_bytes(int64_t n, int d_in, int d_out) {
    if (n < 0 || d_in <= 0 || d_out <= 0) return 0;
    const int splits = std::max(dw_geometry(n, d_in, d_out, GTA_BF16).splits, dw_geometry(n, d_in, d_out, GTA_F32).splits);
    return sizeof(float) * (size_t)splits * (size_t)d_in * (size_t)d_out + 256;   // enough for either element type
}

extern "C" GTA_API size_t gta_linear_dw_group_scratch_bytes(int64_t n, int d_in, int d_out, int p) {
    if (p < 1 || p > 4) return 0;
    return (size_t)p * gta_linear_dw_scratch_bytes(n, d_in, d_out);
}

namespace gta {
namespace {

// p products dW[k] = X[k]^T dY[k] (1 <= p <= 4) of one shape.  bfloat16: one launch for all of them;
// float: one after the other.
gta_status linear_dw_products(const void* const* X, const void* const* dY, float* const* dW, int p, int64_t n,
                              int d_in, int d_out, gta_dtype dtype, void* scratch, size_t scratch_bytes,
                              hipStream_t st) {
    gta_status rc = check_dims(d_in, d_out, dtype);
    if (rc != GTA_OK) return rc;
    if (p < 1 || p > 4) return fail(GTA_ERR_UNSUPPORTED, "1 to 4 products per call, got %d", p);
    if (n < 0) return fail(GTA_ERR_INVALID_ARG, "negative size");
    if (!X || !dY || !dW) return fail(GTA_ERR_INVALID_ARG, "null pointer array");
    for (int k = 0; k < p; ++k) {
        if (!dW[k]) return fail(GTA_ERR_INVALID_ARG, "null tensor pointer");
        if (n > 0 && (!X[k] || !dY[k])) return fail(GTA_ERR_INVALID_ARG, "null tensor pointer");
        if (((uintptr_t)X[k] & 15) || ((uintptr_t)dY[k] & 15))
            return fail(GTA_ERR_INVALID_ARG, "X and dY must be 16-byte aligned");
        for (int m = 0; m < k; ++m)
            if (dW[m] == dW[k]) return fail(GTA_ERR_INVALID_ARG, "products %d and %d name the same result", m, k);
    }
    const size_t need = gta_linear_dw_group_scratch_bytes(n, d_in, d_out, p);
    if (!scratch || scratch_bytes < need) return fail(GTA_ERR_WORKSPACE, "scratch has %zu bytes, %zu needed", scratch_bytes, need);
    const DwGeometry g = dw_geometry(n, d_in, d_out, dtype);
    const int64_t elems = (int64_t)d_in * d_out;
    float* partial = static_cast<float*>(scratch);
    DwResults res{};
    for (int k = 0; k < p; ++k) res.dW[k] = dW[k];
    if (dtype == GTA_F32) {
        for (int k = 0; k < p; ++k) {
            {
                LaunchTimer t("linear_dw", n, 0, st);
                launch_linear_dw_f32((const float*)X[k], (const float*)dY[k], partial, n, d_in, d_out,
                                     g.rows_per_split, g.tiles_i, g.tiles_o, g.splits, st);
            }
            LaunchTimer t("linear_dw.reduce", 0, 0, st);
            DwResults one{};
            one.dW[0] = dW[k];
            hipLaunchKernelGGL(k_reduce_partials, dim3((unsigned)((elems + 31) / 32)), dim3(256), 0, st, partial,
                               one, elems, g.splits);
        }
        GTA_HIP_TRY(hipGetLastError());
        return GTA_OK;
    }
    DwOperands ops{};
    bool shared_x = false;
    for (int k = 0; k < p; ++k) {
        ops.X[k] = (const uint16_t*)X[k];
        ops.dY[k] = (const uint16_t*)dY[k];
        for (int m = 0; m < k; ++m) shared_x = shared_x || X[m] == X[k];
    }
    {
        LaunchTimer t(p == 1 ? "linear_dw" : "linear_dw_group", n, 0, st);
        const int64_t blocks = (int64_t)(g.splits + 7) / 8 * 8 * g.tiles_i * g.tiles_o * p;
#define GTA_LAUNCH_DW(WI, WO, AI, AO, Q, KEEP)                                                                     \
    do {                                                                                                           \
        constexpr size_t lds = dw_lds_bytes<WI, WO, AI, AO>();                                                     \
        GTA_HIP_TRY(hipFuncSetAttribute((const void*)k_linear_dw<WI, WO, AI, AO, Q, KEEP>,                         \
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                    \
        hipLaunchKernelGGL((k_linear_dw<WI, WO, AI, AO, Q, KEEP>), dim3((unsigned)blocks), dim3(64 * WI * WO),     \
                           lds, st, ops, p, partial, n, d_in, d_out, g.rows_per_split, g.tiles_i, g.tiles_o,       \
                           g.splits);                                                                              \
    } while (0)
        if (g.tile == 256 && g.tiles_i == 1 && g.tiles_o == 1) {   // one 256 x 256 tile: the LDS-direct form
            GTA_HIP_TRY(hipFuncSetAttribute((const void*)k_linear_dw_direct<true>,
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDdLdsBytes));
            GTA_HIP_TRY(hipFuncSetAttribute((const void*)k_linear_dw_direct<false>,
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDdLdsBytes));
            if (shared_x)
                hipLaunchKernelGGL(k_linear_dw_direct<true>, dim3((unsigned)blocks), dim3(512), kDdLdsBytes, st, ops, p,
                                   partial, n, d_in, d_out, g.rows_per_split, g.splits);
            else
                hipLaunchKernelGGL(k_linear_dw_direct<false>, dim3((unsigned)blocks), dim3(512), kDdLdsBytes, st, ops, p,
                                   partial, n, d_in, d_out, g.rows_per_split, g.splits);
        } else if (g.tile == 256) {   // 8 wavefronts, each 128 x 64 of a 256 x 256 tile
            if (shared_x) GTA_LAUNCH_DW(2, 4, 4, 2, 2, true); else GTA_LAUNCH_DW(2, 4, 4, 2, 2, false);
        } else {               // 4 wavefronts, each 64 x 64 of the 128 x 128 tile
            if (shared_x) GTA_LAUNCH_DW(2, 2, 2, 2, 4, true); else GTA_LAUNCH_DW(2, 2, 2, 2, 4, false);
        }
#undef GTA_LAUNCH_DW
    }
    {
        LaunchTimer t("linear_dw.reduce", 0, 0, st);
        hipLaunchKernelGGL(k_reduce_partials, dim3((unsigned)((elems + 31) / 32), (unsigned)p), dim3(256), 0, st,
                           partial, res, elems, g.splits);
    }
    GTA_HIP_TRY(hipGetLastError());
    return GTA_OK;
}

}  // namespace
}  // namespace gta

extern "C" GTA_API gta_status gta_linear_dw(const void* X, const void* dY, float* dW, int64_t n, int d_in,
                                            int d_out, gta_dtype dtype, void* scratch, size_t scratch_bytes,
                                            void* stream) {
    return linear_dw_products(&X, &dY, &dW, 1, n, d_in, d_out, dtype, scratch, scratch_bytes,
                              static_cast<hipStream_t>(stream));
}

extern "C" GTA_API gta_status gta_linear_dw_group(const void* const* X, const void* const* dY, float* const* dW,
                                                  int p, int64_t n, int d_in, int d_out, gta_dtype dtype,
                                                  void* scratch, size_t scratch_bytes, void* stream) {
    return linear_dw_products(X, dY, dW, p, n, d_in, d_out, dtype, scratch, scratch_bytes,
                              static_cast<hipStream_t>(stream));
}
