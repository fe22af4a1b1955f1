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

constexpr int kProjThreads = 512, kProjRows = 128, kProjKC = 32, kProjWPitch = kProjKC + 8;
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
// Wp[(m * KCH + kc) * D + col][kk] = W_m(k = 32 kc + kk, col), where W_m(k, col) is W_m[k * D + col]
// (trans = 0: stored [d_in, d_out]) or W_m[col * D + k] (trans = 1: stored [d_out, d_in]).
struct PackArgs { const uint16_t* W[kProjMaxParts * kProjMaxParts]; };
__global__ void __launch_bounds__(256) k_pack_weights(PackArgs a, uint16_t* __restrict__ Wp, int D, int mats, int trans) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t per = (int64_t)D * D;
    if (e >= per * mats) return;
    const int m = (int)(e / per);
    const int r = (int)(e - m * per);
    const int kk = r % kProjKC, col = (r / kProjKC) % D, kc = r / (kProjKC * D);
    const int k = kc * kProjKC + kk;
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

template <int D, int P_IN, int P_OUT, bool HAS_C>
__global__ void __launch_bounds__(kProjThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_proj(ProjArgs a) {
    using S = ProjShape<D>;
    constexpr int CT = S::CT, RT = S::RT, XPitch = S::XPitch, PPitch = S::PPitch, KCH = S::KCH;
    constexpr int WPitch = kProjWPitch;
    // Global loads are split by wavefront: wavefronts 0-3 fetch the weight chunks, wavefronts 4-7 the X tiles
    // (and every wavefront multiplies).  A wavefront's loads complete in order, so a wavefront that had an
    // X tile (HBM latency) in flight would have to sit it out at its next wait for a weight chunk (L2 latency).
    constexpr int kLoaders = kProjThreads / 2;
    constexpr int XUnitsPerRow = D / 8, XU = kProjRows * XUnitsPerRow / kLoaders;   // X tile units per loading thread
    constexpr int WUnits = D * (kProjKC / 8);                                      // units of a weight chunk
    constexpr int WU = WUnits / kLoaders;
    static_assert(WUnits % kLoaders == 0 && (kProjRows * XUnitsPerRow) % kLoaders == 0, "whole units per loader");
    constexpr int UPR = 4 * CT, RPI = 64 / UPR, NI = 32 / RPI;   // result patch: units per row, rows per instruction
    constexpr int TOTAL_CHUNKS = P_OUT * P_IN * KCH;
    extern __shared__ __align__(16) unsigned char proj_lds[];
    uint16_t* xs = reinterpret_cast<uint16_t*>(proj_lds);        // [128][XPitch]
    uint16_t* ws = xs + kProjRows * XPitch;                      // [2][D][WPitch]
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, g = lane >> 5, r32 = lane & 31;
    const int wr = w / S::WAVES_C, wc = w % S::WAVES_C;
    const bool loads_w = w < 4;                     // wave-uniform role
    const unsigned lt = (unsigned)tid & (kLoaders - 1);   // index among the threads of the same role
    uint16_t* patch = ws + 2 * D * WPitch + w * (32 * PPitch);   // this wavefront's [32][PPitch]
    const int crow = lane / UPR, cunit = lane % UPR;             // this lane's unit of a patch row group
    const int col0 = wc * CT * 32;                               // first column of this wavefront

    u32x4 xregs[XU], wregs[2][WU], cregs[HAS_C ? RT * NI : 1];
    // Global addresses are a per-block base (uniform, kept in scalar registers) plus a 32-bit element
    // offset inside the block's 128 x D window; rows past the end of the tensor are clamped to its last
    // row.  (64-bit per-thread addresses for every load would not fit the register budget.)
    auto rows_in_block = [&](int64_t rb) {   // valid rows of block rb, at least 1
        const int64_t left = a.n - rb * kProjRows;
        return (int)(left < kProjRows ? left : kProjRows);
    };
    auto load_x = [&](int64_t rb, int pi) {   // X_pi rows of block rb -> registers
        if (loads_w) return;
        const char* base = reinterpret_cast<const char*>(a.X[pi] + rb * (kProjRows * D));
        const unsigned lim = (unsigned)rows_in_block(rb) - 1u;
#pragma unroll
        for (int i = 0; i < XU; ++i) {
            const unsigned u = lt + i * kLoaders, r = u / XUnitsPerRow, cu = u % XUnitsPerRow;
            const unsigned off = ((r < lim ? r : lim) * D + cu * 8) * 2u;   // bytes
            xregs[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + off));
        }
    };
    auto store_x = [&]() {
        if (loads_w) return;
#pragma unroll
        for (int i = 0; i < XU; ++i) {
            const unsigned u = lt + i * kLoaders, r = u / XUnitsPerRow, cu = u % XUnitsPerRow;
            *reinterpret_cast<u32x4*>(xs + r * XPitch + cu * 8) = xregs[i];
        }
    };
    auto load_w = [&](int set, int ci) {      // packed chunk ci -> register set `set`
        if (!loads_w) return;
        const char* src = reinterpret_cast<const char*>(a.Wp + (int64_t)ci * (D * kProjKC));
#pragma unroll
        for (int i = 0; i < WU; ++i) {
            const unsigned u = lt + i * kLoaders;
            wregs[set][i] = *reinterpret_cast<const u32x4*>(src + u * 16u);
        }
    };
    auto store_w = [&](int set, int buf) {
        if (!loads_w) return;
        uint16_t* dst = ws + buf * (D * WPitch);
#pragma unroll
        for (int i = 0; i < WU; ++i) {
            const unsigned u = lt + i * kLoaders;
            *reinterpret_cast<u32x4*>(dst + (u >> 2) * WPitch + (u & 3) * 8) = wregs[set][i];
        }
    };
    auto wrap = [](int ci) { return ci >= TOTAL_CHUNKS ? ci - TOTAL_CHUNKS : ci; };
    auto load_c = [&](int64_t rb, int po) {   // this wavefront's tile of the addend, in patch-row order
        if constexpr (HAS_C) {
            const char* base = reinterpret_cast<const char*>(a.C[po] + rb * (kProjRows * D));
            const unsigned lim = (unsigned)rows_in_block(rb) - 1u;
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int q = 0; q < NI; ++q) {
                    const unsigned r = (unsigned)((wr * RT + rt) * 32 + RPI * q + crow);
                    const unsigned off = ((r < lim ? r : lim) * D + (unsigned)(col0 + 8 * cunit)) * 2u;
                    cregs[rt * NI + q] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + off));
                }
        }
    };

    floatx16 acc[RT][CT];
    auto zero_acc = [&]() {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[rt][ct][v] = 0.f;
    };
    auto compute = [&](int kc, int buf) {     // one weight chunk: two k steps of 16
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
    };
    // rounds the wavefront's tiles (after adding the addend), lays each 32-row group out row-major in
    // the patch and stores it in whole 16-byte units; rows past the end are not stored
    auto epilogue = [&](int64_t rb, int po) {
        char* ybase = reinterpret_cast<char*>(a.Y[po] + rb * (kProjRows * D));
        const int valid = rows_in_block(rb);
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
                if (r < valid)
                    __builtin_nontemporal_store(
                        *reinterpret_cast<const u32x4*>(patch + (RPI * q + crow) * PPitch + 8 * cunit),
                        reinterpret_cast<u32x4*>(ybase + (unsigned)(r * D + col0 + 8 * cunit) * 2u));
            }
        }
    };

    int64_t rb = blockIdx.x;
    if (rb >= a.row_blocks) return;   // whole workgroup leaves together
    // The weight chunks run two ahead: while chunk c is multiplied out of LDS buffer c % 2, chunk c + 1
    // sits in a register set (fetched during chunk c - 1, stored to the other buffer after the
    // multiplication) and chunk c + 2 is being fetched into the other set, so an L2 round trip has
    // two chunks' worth of matrix work to hide behind.  Chunk parity = buffer = register set, which
    // the loop unrolled by two keeps static (every product has an even number of chunks).
    static_assert(KCH % 2 == 0, "chunks per product");
    load_x(rb, 0);
    load_w(0, 0);
    store_x();
    store_w(0, 0);
    load_w(1, wrap(1));
    __syncthreads();
    int ci = 0;   // chunk being multiplied (always even at the top of the unrolled pair)
    for (; rb < a.row_blocks; rb += gridDim.x) {
        // the block after this one (when there is none: this one again, fetched and never used)
        const int64_t next_rb = rb + gridDim.x < a.row_blocks ? rb + gridDim.x : rb;
#pragma unroll
        for (int po = 0; po < P_OUT; ++po) {
            zero_acc();
#pragma unroll
            for (int pi = 0; pi < P_IN; ++pi) {
                const bool last_of_block = po == P_OUT - 1 && pi == P_IN - 1;
                // the X tile changes after this product unless the next product reads the same input
                constexpr bool shared_x = P_IN == 1;
                const bool swap_x = !shared_x || po == P_OUT - 1;
                if (swap_x) load_x(last_of_block ? next_rb : rb, (pi + 1) % P_IN);
                if (pi == P_IN - 1) load_c(rb, po);
#pragma unroll 1
                for (int kc = 0; kc < KCH; kc += 2) {
                    load_w(0, wrap(ci + 2));
                    __builtin_amdgcn_sched_barrier(0);   // the fetch is issued before the multiplication, not after
                    compute(kc, 0);
                    store_w(1, 1);      // buffer 1 was last read during the previous chunk, before its barrier
                    __syncthreads();
                    load_w(1, wrap(ci + 3));
                    __builtin_amdgcn_sched_barrier(0);
                    compute(kc + 1, 1);
                    store_w(0, 0);
                    __syncthreads();
                    ci = wrap(ci + 2);
                }
                if (swap_x) store_x();  // every wavefront has passed the last chunk's barrier: the tile is free
                if (pi == P_IN - 1) epilogue(rb, po);
                if (swap_x) __syncthreads();
            }
        }
    }
}

template <int D, int P_IN, int P_OUT, bool HAS_C>
gta_status launch_proj(const ProjArgs& a, hipStream_t st) {
    constexpr size_t lds = ProjShape<D>::lds_bytes;
    GTA_HIP_TRY(hipFuncSetAttribute((const void*)k_proj<D, P_IN, P_OUT, HAS_C>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    int device = 0, cus = 0;
    GTA_HIP_TRY(hipGetDevice(&device));
    GTA_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device));
    if (cus <= 0) cus = 256;
    const int64_t blocks = a.row_blocks < cus ? a.row_blocks : cus;
    hipLaunchKernelGGL((k_proj<D, P_IN, P_OUT, HAS_C>), dim3((unsigned)blocks), dim3(kProjThreads), lds, st, a);
    GTA_HIP_TRY(hipGetLastError());
    return GTA_OK;
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
