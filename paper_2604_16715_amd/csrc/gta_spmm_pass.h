// SpMM pass over per-entry weights: Y[row] = out_scale * sum_e W[e,h] * X[col(e)].  Used by the
// standalone gta_spmm operator and by the backward's dQ = dZ K step (Section 2.2).
#pragma once
#include "gta_kernels.h"

namespace gta {

template <class T, int LH_, int G_>
struct SpmmPass {
    static constexpr int LH = LH_, G = G_, U = UnrollFor<G_>::value;
    static constexpr int NV = Elt<T>::NV;
    static constexpr bool kUsesEntryId = true;
    static constexpr int N = NV;
    struct Params {
        const float* Wt;
        SegConst X;   // gathered by column id
        int split;
        char* Y;
        float* partial;
        int64_t stride;
        float out_scale;
        int heads;
    };
    float f[N];
    uint4 xr[U];
    float w[U];

    __device__ __forceinline__ void init(const Params&, int, int, bool, bool) {
#pragma unroll
        for (int i = 0; i < N; ++i) f[i] = 0.f;
    }
    __device__ __forceinline__ void load(const Params& p, int u, int j, int e, bool ok, int lig) {
        xr[u] = make_uint4(0, 0, 0, 0);
        w[u] = 0.f;
        if (ok) {
            xr[u] = load16(p.X, p.split, j, p.stride, lig);
            w[u] = __builtin_nontemporal_load(p.Wt + (int64_t)e * p.heads + lig / LH);   // every weight is read once
        }
    }
    __device__ __forceinline__ void compute(const bool (&)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float x[NV];
            Elt<T>::unpack(xr[u], x);
#pragma unroll
            for (int i = 0; i < NV; ++i) f[i] = fmaf(w[u], x[i], f[i]);
        }
    }
    static __device__ __forceinline__ void combine(float (&a)[N], const float (&b)[N]) {
#pragma unroll
        for (int i = 0; i < N; ++i) a[i] += b[i];
    }
    static __device__ __forceinline__ void finish(const Params& p, int row, int lig, const float (&a)[N]) {
        float o[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) o[i] = a[i] * p.out_scale;
        store16(p.Y, row, p.stride, lig, Elt<T>::pack(o));
    }
};

}  // namespace gta
