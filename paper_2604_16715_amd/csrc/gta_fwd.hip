// Forward pass: Eq. 4-5 fused.  Per stored entry the score s = q_i . k_j / sqrt(d) (SDDMM), the
// row softmax evaluated online (running maximum m and sum l, accumulator rescaled when the
// maximum moves), and the weighted sum of value rows (SpMM).  Scores are kept in base 2
// (pre-multiplied by log2 e) so the exponential is one v_exp_f32.
#include "gta_kernels.h"

namespace gta {
namespace {

template <class T, int LH_, int G_>
struct FwdPass {
    static constexpr int LH = LH_, G = G_, U = UnrollFor<G_>::value;
    static constexpr int NV = Elt<T>::NV;
    static constexpr bool kUsesEntryId = false;
    static constexpr int N = NV + 2;   // f = accumulator[NV], running max, running sum
    struct Params {
        const char* Q;
        SegConst K, V;
        int split;
        char* out;
        float* lse;
        float* partial;
        int64_t stride;
        float qscale;   // scale * log2(e)
        int heads;
    };
    uint4 q;         // this lane's 16 bytes of the query row, as stored
    float qscale;
    float f[N];
    uint4 kr[U], vr[U];

    __device__ __forceinline__ void init(const Params& p, int row, int lig, bool active, bool) {
#pragma unroll
        for (int i = 0; i < NV; ++i) f[i] = 0.f;
        f[NV] = kNegBig;
        f[NV + 1] = 0.f;
        qscale = p.qscale;
        q = make_uint4(0, 0, 0, 0);
        if (active) q = load16_stream(p.Q, row, p.stride, lig);
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
        float s[U];
        float mn = f[NV];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float d = head_allreduce<LH>(Elt<T>::dot(q, kr[u])) * qscale;
            s[u] = ok[u] ? d : -INFINITY;
            mn = fmaxf(mn, s[u]);
        }
        const float corr = fast_exp2(f[NV] - mn);
        float lsum = f[NV + 1] * corr;
#pragma unroll
        for (int i = 0; i < NV; ++i) f[i] *= corr;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float pw = fast_exp2(s[u] - mn);
            lsum += pw;
            float v[NV];
            Elt<T>::unpack(vr[u], v);
#pragma unroll
            for (int i = 0; i < NV; ++i) f[i] = fmaf(pw, v[i], f[i]);
        }
        f[NV] = mn;
        f[NV + 1] = lsum;
    }
    static __device__ __forceinline__ void combine(float (&a)[N], const float (&b)[N]) {
        const float mn = fmaxf(a[NV], b[NV]);
        const float ca = fast_exp2(a[NV] - mn), cb = fast_exp2(b[NV] - mn);
#pragma unroll
        for (int i = 0; i < NV; ++i) a[i] = a[i] * ca + b[i] * cb;
        a[NV + 1] = a[NV + 1] * ca + b[NV + 1] * cb;
        a[NV] = mn;
    }
    static __device__ __forceinline__ void finish(const Params& p, int row, int lig, const float (&a)[N]) {
        const float l = a[NV + 1];
        const float inv = l > 0.f ? 1.0f / l : 0.f;
        float o[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) o[i] = a[i] * inv;
        store16(p.out, row, p.stride, lig, Elt<T>::pack(o));
        if (lig % LH == 0)
            p.lse[(int64_t)row * p.heads + lig / LH] = l > 0.f ? (a[NV] + fast_log2(l)) * kLn2 : -INFINITY;
    }
};

template <class T> gta_status run(const AttnArgs& a) {
    const Shape& sh = a.shape;
#define GTA_CALL(LHc, Gc)                                                                             \
    {                                                                                                 \
        using P = FwdPass<T, LHc, Gc>;                                                                \
        typename P::Params prm{(const char*)a.Q, seg_of(a, a.K, a.K_halo), seg_of(a, a.V, a.V_halo),  \
                               seg_split(a), (char*)a.o_out,                                          \
                               a.lse_out, a.partial, sh.row_bytes, a.scale * kLog2e, sh.heads};       \
        return launch_pass<P>("fwd", prm, a.plan, 0, nullptr, a.stream);                                       \
    }
    GTA_DISPATCH_GEOMETRY(sh.lanes_per_head, sh.lanes_per_row, GTA_CALL)
#undef GTA_CALL
    return GTA_OK;
}

}  // namespace

gta_status launch_fwd(const AttnArgs& a) {
    return a.shape.elem_bytes == 4 ? run<float>(a) : run<bf16_tag>(a);
}

}  // namespace gta
