// Backward, destination-major pass (Section 2.2): for every stored entry of row i the weight is
// recomputed from the saved log-sum-exp, a = exp(s - lse); then
//     dU = dY_i . v_j                       (the backward SDDMM)
//     dZ = a * (dU - delta_i)               (softmax backward, delta_i = sum_e a_e dU_e = dY_i . Y_i)
//     dQ_i += scale * dZ * k_j              (SpMM dQ = dZ K)
// It also leaves (lse * log2 e, delta) per (row, head) for the source-major pass.
//
// Second form, used when the caller's scratch can hold dZ for every stored entry: a streaming
// kernel writes (lse * log2 e, delta) first, the source-major pass computes dZ and stores it in
// transposed order, and dQ is then a plain SpMM over the stored dZ that gathers K only (one row
// gather per entry less).
#include "gta_kernels.h"
#include "gta_spmm_pass.h"

namespace gta {
namespace {

template <class T, int LH_, int G_>
struct BwdDstPass {
    static constexpr int LH = LH_, G = G_, U = UnrollFor<G_>::value;
    static constexpr int NV = Elt<T>::NV;
    static constexpr bool kUsesEntryId = false;
    static constexpr int N = NV;   // f = dQ accumulator (unscaled)
    struct Params {
        const char* Q;
        SegConst K, V;
        int split;
        const char *out, *dO;
        char* dQ;
        const float* lse;
        float2* rowstat;
        float* partial;
        int64_t stride;
        float qscale, scale;
        int heads;
    };
    uint4 qraw, graw;   // this lane's 16 bytes of the row's query and output-gradient, as stored
    float qscale;
    float lse2, delta;
    float f[N];
    uint4 kr[U], vr[U];

    __device__ __forceinline__ void init(const Params& p, int row, int lig, bool active, bool primary) {
#pragma unroll
        for (int i = 0; i < NV; ++i) f[i] = 0.f;
        lse2 = 0.f;
        delta = 0.f;
        qscale = p.qscale;
        qraw = make_uint4(0, 0, 0, 0);
        graw = make_uint4(0, 0, 0, 0);
        if (active) {
            qraw = load16(p.Q, row, p.stride, lig);
            graw = load16(p.dO, row, p.stride, lig);
            delta = Elt<T>::dot(graw, load16(p.out, row, p.stride, lig));
            lse2 = p.lse[(int64_t)row * p.heads + lig / LH] * kLog2e;
        }
        delta = head_allreduce<LH>(delta);
        if (active && primary && lig % LH == 0)
            p.rowstat[(int64_t)row * p.heads + lig / LH] = make_float2(lse2, delta);
    }
    __device__ __forceinline__ void load(const Params& p, int u, int j, int, bool ok, int lig) {
        kr[u] = make_uint4(0, 0, 0, 0);
        vr[u] = make_uint4(0, 0, 0, 0);
        if (ok) {
            kr[u] = load16(p.K, p.split, j, p.stride, lig);
            vr[u] = load16(p.V, p.split, j, p.stride, lig);
        }
    }
    __device__ __forceinline__ void compute(const bool (&ok)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float k[NV];
            Elt<T>::unpack(kr[u], k);
            const float s = head_allreduce<LH>(Elt<T>::dot(qraw, kr[u])) * qscale;
            const float da = head_allreduce<LH>(Elt<T>::dot(graw, vr[u]));
            const float a = ok[u] ? fast_exp2(s - lse2) : 0.f;
            const float dz = a * (da - delta);
#pragma unroll
            for (int i = 0; i < NV; ++i) f[i] = fmaf(dz, k[i], f[i]);
        }
    }
    static __device__ __forceinline__ void combine(float (&a)[N], const float (&b)[N]) {
#pragma unroll
        for (int i = 0; i < N; ++i) a[i] += b[i];
    }
    static __device__ __forceinline__ void finish(const Params& p, int row, int lig, const float (&a)[N]) {
        float o[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) o[i] = a[i] * p.scale;
        store16(p.dQ, row, p.stride, lig, Elt<T>::pack(o));
    }
};

// one group of G lanes per destination row, rows in natural order
template <class T, int LH, int G>
__global__ void __launch_bounds__(kBlockThreads)
k_rowstat(const char* out, const char* dO, const float* lse, float2* rowstat, int64_t n_rows, int64_t stride,
          int heads) {
    const int64_t row = ((int64_t)blockIdx.x * kBlockThreads + threadIdx.x) / G;
    const int lig = threadIdx.x % G;
    float d = 0.f;
    if (row < n_rows) {
        d = Elt<T>::dot(load16_stream(dO, row, stride, lig), load16_stream(out, row, stride, lig));
    }
    d = head_allreduce<LH>(d);
    if (row < n_rows && lig % LH == 0)
        rowstat[row * heads + lig / LH] = make_float2(lse[row * heads + lig / LH] * kLog2e, d);
}

template <class T> gta_status run_rowstat(const AttnArgs& a) {
    const Shape& sh = a.shape;
    const int64_t n = a.plan->n_dst;
#define GTA_CALL(LHc, Gc)                                                                            \
    {                                                                                                \
        const int64_t blocks = (n * Gc + kBlockThreads - 1) / kBlockThreads;                         \
        LaunchTimer t("bwd_rowstat", n, 0, a.stream);                                                \
        hipLaunchKernelGGL((k_rowstat<T, LHc, Gc>), dim3((unsigned)blocks), dim3(kBlockThreads), 0,  \
                           a.stream, (const char*)a.out, (const char*)a.dO, a.lse_in, a.rowstat, n,  \
                           sh.row_bytes, sh.heads);                                                  \
    }
    GTA_DISPATCH_GEOMETRY(sh.lanes_per_head, sh.lanes_per_row, GTA_CALL)
#undef GTA_CALL
    GTA_HIP_TRY(hipGetLastError());
    return GTA_OK;
}

template <class T> gta_status run_dq(const AttnArgs& a) {
    const Shape& sh = a.shape;
#define GTA_CALL(LHc, Gc)                                                                            \
    {                                                                                                \
        using P = SpmmPass<T, LHc, Gc>;                                                              \
        typename P::Params prm{a.dS, seg_of(a, a.K, a.K_halo), seg_split(a), (char*)a.dQ, a.partial, \
                               sh.row_bytes, a.scale, sh.heads};                                     \
        return launch_pass<P>("bwd_dq", prm, a.plan, 0, a.plan->t_pos, a.stream);                                   \
    }
    GTA_DISPATCH_GEOMETRY(sh.lanes_per_head, sh.lanes_per_row, GTA_CALL)
#undef GTA_CALL
    return GTA_OK;
}

template <class T> gta_status run(const AttnArgs& a) {
    const Shape& sh = a.shape;
#define GTA_CALL(LHc, Gc)                                                                            \
    {                                                                                                \
        using P = BwdDstPass<T, LHc, Gc>;                                                            \
        typename P::Params prm{(const char*)a.Q, seg_of(a, a.K, a.K_halo), seg_of(a, a.V, a.V_halo), \
                               seg_split(a),                                                         \
                               (const char*)a.out, (const char*)a.dO, (char*)a.dQ, a.lse_in,         \
                               a.rowstat, a.partial, sh.row_bytes, a.scale * kLog2e, a.scale,        \
                               sh.heads};                                                            \
        return launch_pass<P>("bwd_dst", prm, a.plan, 0, nullptr, a.stream);                                  \
    }
    GTA_DISPATCH_GEOMETRY(sh.lanes_per_head, sh.lanes_per_row, GTA_CALL)
#undef GTA_CALL
    return GTA_OK;
}

}  // namespace

gta_status launch_rowstat(const AttnArgs& a) {
    return a.shape.elem_bytes == 4 ? run_rowstat<float>(a) : run_rowstat<bf16_tag>(a);
}

gta_status launch_bwd_dq(const AttnArgs& a) {
    return a.shape.elem_bytes == 4 ? run_dq<float>(a) : run_dq<bf16_tag>(a);
}

gta_status launch_bwd_dst(const AttnArgs& a) {
    return a.shape.elem_bytes == 4 ? run<float>(a) : run<bf16_tag>(a);
}

}  // namespace gta
