// Backward, source-major pass (Section 2.2): the two SpMMs with the transposed adjacency,
//     dV_j = sum_{i : j in N(i)} a_ij * dY_i          (dV = U^T dY)
//     dK_j = sum_{i : j in N(i)} scale * dZ_ij * q_i   (dK = dZ^T Q)
// walked over the plan's transposed pattern so each source row is owned by one group of lanes
// and summed in a fixed order (no atomics).  Per entry the weight a_ij and dZ_ij are recomputed
// from q_i, dY_i and the (lse, delta) pair of row i.  With STORE the pass also writes dZ_ij
// (unscaled) to a float [nnz, heads] array in the order it walks (transposed order, so the writes
// are contiguous); dQ = dZ K afterwards runs as a plain SpMM that gathers only K and finds each
// entry's dZ through the plan's stored-position -> transposed-position map.
#include "gta_kernels.h"

namespace gta {
namespace {

template <class T, int LH_, int G_, bool STORE>
struct BwdSrcPass {
    static constexpr int LH = LH_, G = G_, U = UnrollFor<G_>::value;
    static constexpr int NV = Elt<T>::NV;
    static constexpr bool kUsesEntryId = STORE;
    static constexpr int N = 2 * NV;   // f = dK accumulator (unscaled), then dV accumulator
    struct Params {
        const char *Q, *dO;
        SegConst K, V;   // read by the row that owns them
        SegMut dK, dV;
        int split;
        const float2* rowstat;
        float* dS;
        float* partial;
        int64_t stride;
        float qscale, scale;
        int heads;
    };
    uint4 kraw, vraw;   // this lane's 16 bytes of the source's key and value rows, as stored
    float qscale;
    float f[N];
    uint4 qr[U], gr[U];
    float2 st[U];
    int eids[U];
    float* ds_out;
    int n_heads, my_lig;

    __device__ __forceinline__ void init(const Params& p, int row, int lig, bool active, bool) {
#pragma unroll
        for (int i = 0; i < NV; ++i) { f[i] = 0.f; f[NV + i] = 0.f; }
        kraw = make_uint4(0, 0, 0, 0);
        vraw = make_uint4(0, 0, 0, 0);
        qscale = p.qscale;
        ds_out = p.dS;
        n_heads = p.heads;
        my_lig = lig;
        if (active) {
            kraw = load16_stream(row < p.split ? p.K.lo : p.K.hi, row, p.stride, lig);   // its owner reads it once
            vraw = load16_stream(row < p.split ? p.V.lo : p.V.hi, row, p.stride, lig);
        }
    }
    __device__ __forceinline__ void load(const Params& p, int u, int i, int e, bool ok, int lig) {
        eids[u] = e;
        qr[u] = make_uint4(0, 0, 0, 0);
        gr[u] = make_uint4(0, 0, 0, 0);
        st[u] = make_float2(0.f, 0.f);
        if (ok) {
            qr[u] = load16(p.Q, i, p.stride, lig);
            gr[u] = load16(p.dO, i, p.stride, lig);
            st[u] = p.rowstat[(int64_t)i * p.heads + lig / LH];
        }
    }
    __device__ __forceinline__ void compute(const bool (&ok)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float q[NV], go[NV];
            Elt<T>::unpack(qr[u], q);
            Elt<T>::unpack(gr[u], go);
            const float s = head_allreduce<LH>(Elt<T>::dot(qr[u], kraw)) * qscale;
            const float da = head_allreduce<LH>(Elt<T>::dot(gr[u], vraw));
            const float a = ok[u] ? fast_exp2(s - st[u].x) : 0.f;
            const float dz = a * (da - st[u].y);
            if (STORE && ok[u] && my_lig % LH == 0) __builtin_nontemporal_store(dz, ds_out + (int64_t)eids[u] * n_heads + my_lig / LH);
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                f[i] = fmaf(dz, q[i], f[i]);
                f[NV + i] = fmaf(a, go[i], f[NV + i]);
            }
        }
    }
    static __device__ __forceinline__ void combine(float (&a)[N], const float (&b)[N]) {
#pragma unroll
        for (int i = 0; i < N; ++i) a[i] += b[i];
    }
    static __device__ __forceinline__ void finish(const Params& p, int row, int lig, const float (&a)[N]) {
        float dk[NV], dv[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) { dk[i] = a[i] * p.scale; dv[i] = a[NV + i]; }
        store16(p.dK, p.split, row, p.stride, lig, Elt<T>::pack(dk));
        store16(p.dV, p.split, row, p.stride, lig, Elt<T>::pack(dv));
    }
};

template <class T, bool STORE> gta_status run(const AttnArgs& a) {
    const Shape& sh = a.shape;
#define GTA_CALL(LHc, Gc)                                                                         \
    {                                                                                             \
        using P = BwdSrcPass<T, LHc, Gc, STORE>;                                                  \
        typename P::Params prm{(const char*)a.Q, (const char*)a.dO, seg_of(a, a.K, a.K_halo),     \
                               seg_of(a, a.V, a.V_halo), seg_of(a, a.dK, a.dK_halo),              \
                               seg_of(a, a.dV, a.dV_halo), seg_split(a), a.rowstat, a.dS,         \
                               a.partial, sh.row_bytes, a.scale * kLog2e, a.scale, sh.heads};     \
        return launch_pass<P>("bwd_src", prm, a.plan, 1, nullptr, a.stream);                               \
    }
    GTA_DISPATCH_GEOMETRY(sh.lanes_per_head, sh.lanes_per_row, GTA_CALL)
#undef GTA_CALL
    return GTA_OK;
}

}  // namespace

gta_status launch_bwd_src(const AttnArgs& a) {
    if (a.dS) return a.shape.elem_bytes == 4 ? run<float, true>(a) : run<bf16_tag, true>(a);
    return a.shape.elem_bytes == 4 ? run<float, false>(a) : run<bf16_tag, false>(a);
}

}  // namespace gta
