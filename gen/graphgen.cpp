// Seeded synthetic input generators: power-law / R-MAT graphs in CSR-by-destination form and
// N(0,1) tensors.  This module serves both the CPU oracle's tests and the GPU path's tests and
// benchmark.  It contains no attention arithmetic: only a counter-based random number
// generator, graph sampling, CSR assembly and storage-format rounding of the *inputs*.
//
// Everything is a pure function of (seed, stream, index), so results do not depend on the
// number of OpenMP threads.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <numeric>
#include <vector>
#include <omp.h>

namespace {

inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// counter-based generator: one 64-bit word per (seed, stream, index)
inline uint64_t rnd_u64(uint64_t seed, uint64_t stream, uint64_t index) {
    uint64_t k = mix64(seed ^ mix64(stream * 0xD1342543DE82EF95ull + 0x2545F4914F6CDD1Dull));
    return mix64(k ^ mix64(index));
}

// uniform in the open interval (0,1)
inline double rnd_unit(uint64_t seed, uint64_t stream, uint64_t index) {
    return ((double)(rnd_u64(seed, stream, index) >> 11) + 0.5) * (1.0 / 9007199254740992.0);
}

// seeded bijection of [0,n): order of hashed keys
void make_permutation(std::vector<int32_t>& perm, int64_t n, uint64_t seed, uint64_t stream) {
    std::vector<std::pair<uint64_t, int32_t>> keyed((size_t)n);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) keyed[(size_t)i] = {rnd_u64(seed, stream, (uint64_t)i), (int32_t)i};
    std::sort(keyed.begin(), keyed.end());
    perm.resize((size_t)n);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) perm[(size_t)i] = keyed[(size_t)i].second;
}

// Assemble CSR-by-destination from (dst,src) pairs: per-row sort by source, duplicates dropped.
// Returns the number of stored entries.  indices must have room for pairs.size() entries.
int64_t build_csr(const std::vector<int32_t>& dst, const std::vector<int32_t>& src, int64_t n_dst,
                  int64_t* indptr, int32_t* indices) {
    const int64_t m = (int64_t)dst.size();
    std::vector<int64_t> start((size_t)n_dst + 1, 0);
    for (int64_t e = 0; e < m; ++e) start[(size_t)dst[(size_t)e] + 1]++;
    for (int64_t i = 0; i < n_dst; ++i) start[(size_t)i + 1] += start[(size_t)i];
    std::vector<int32_t> bucket((size_t)m);
    {
        std::vector<int64_t> cursor(start.begin(), start.end() - 1);
        for (int64_t e = 0; e < m; ++e) bucket[(size_t)cursor[(size_t)dst[(size_t)e]]++] = src[(size_t)e];
    }
    std::vector<int64_t> uniq((size_t)n_dst + 1, 0);
#pragma omp parallel for schedule(dynamic, 1024)
    for (int64_t i = 0; i < n_dst; ++i) {
        int32_t* b = bucket.data() + start[(size_t)i];
        int32_t* e = bucket.data() + start[(size_t)i + 1];
        std::sort(b, e);
        uniq[(size_t)i + 1] = std::unique(b, e) - b;
    }
    indptr[0] = 0;
    for (int64_t i = 0; i < n_dst; ++i) indptr[i + 1] = indptr[i] + uniq[(size_t)i + 1];
#pragma omp parallel for schedule(dynamic, 1024)
    for (int64_t i = 0; i < n_dst; ++i)
        std::memcpy(indices + indptr[i], bucket.data() + start[(size_t)i],
                    (size_t)(indptr[i + 1] - indptr[i]) * sizeof(int32_t));
    return indptr[n_dst];
}

// sum over r in [0,n) of (r + r0)^expo, in fixed blocks so the result does not depend on threads
double weight_sum(int64_t n, double r0, double expo) {
    const int64_t blk = 1 << 16, nb = (n + blk - 1) / blk;
    std::vector<double> part((size_t)nb);
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < nb; ++b) {
        double acc = 0.0;
        const int64_t hi = std::min(n, (b + 1) * blk);
        for (int64_t r = b * blk; r < hi; ++r) acc += std::pow((double)r + r0, expo);
        part[(size_t)b] = acc;
    }
    double tot = 0.0;
    for (int64_t b = 0; b < nb; ++b) tot += part[(size_t)b];
    return tot;
}

// cumulative distribution of rank weights w_r = (r + r0)^(-1/(gamma-1)), r = 0..n-1
void rank_cdf(std::vector<double>& cdf, int64_t n, double gamma, double r0) {
    cdf.resize((size_t)n);
    const double expo = -1.0 / (gamma - 1.0);
    double acc = 0.0;
    for (int64_t r = 0; r < n; ++r) {
        acc += std::pow((double)r + r0, expo);
        cdf[(size_t)r] = acc;
    }
    for (int64_t r = 0; r < n; ++r) cdf[(size_t)r] /= acc;
    cdf[(size_t)n - 1] = 1.0;
}

// r0 such that the heaviest rank expects `target` of `draws` samples (bisection on r0)
double solve_r0(int64_t n, double gamma, double draws, double target) {
    const double expo = -1.0 / (gamma - 1.0);
    double lo = 1e-3, hi = (double)n;
    for (int it = 0; it < 48; ++it) {
        double mid = std::sqrt(lo * hi);
        double share = std::pow(mid, expo) / weight_sum(n, mid, expo);
        if (share * draws > target) lo = mid; else hi = mid;
    }
    return std::sqrt(lo * hi);
}

inline int64_t sample_rank(const std::vector<double>& cdf, double u) {
    return (int64_t)(std::lower_bound(cdf.begin(), cdf.end(), u) - cdf.begin());
}

inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

}  // namespace

extern "C" {

// Chung-Lu style power-law graph.  `draws` (dst,src) pairs are sampled with independent
// rank->node maps for the in- and out-weights; with symmetric != 0 every draw stores both
// directions.  One self-loop is added per node, then rows are sorted and deduplicated.
// indices must have room for draws*(symmetric?2:1) + n entries.  Returns realised nnz.
int64_t gen_chung_lu(int64_t n, int64_t draws, double gamma, double target_max_deg, int symmetric,
                     uint64_t seed, int64_t* indptr, int32_t* indices) {
    const double eff_draws = symmetric ? 2.0 * (double)draws : (double)draws;
    const double r0 = solve_r0(n, gamma, eff_draws, target_max_deg);
    std::vector<double> cdf;
    rank_cdf(cdf, n, gamma, r0);
    std::vector<int32_t> map_in, map_out;
    make_permutation(map_in, n, seed, 6);
    if (symmetric) map_out = map_in; else make_permutation(map_out, n, seed, 7);
    const int64_t per = symmetric ? 2 : 1;
    std::vector<int32_t> dst((size_t)(draws * per + n)), src((size_t)(draws * per + n));
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < draws; ++t) {
        int32_t a = map_in[(size_t)sample_rank(cdf, rnd_unit(seed, 0, (uint64_t)t))];
        int32_t b = map_out[(size_t)sample_rank(cdf, rnd_unit(seed, 1, (uint64_t)t))];
        dst[(size_t)(t * per)] = a;
        src[(size_t)(t * per)] = b;
        if (symmetric) {
            dst[(size_t)(t * per + 1)] = b;
            src[(size_t)(t * per + 1)] = a;
        }
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        dst[(size_t)(draws * per + i)] = (int32_t)i;
        src[(size_t)(draws * per + i)] = (int32_t)i;
    }
    return build_csr(dst, src, n, indptr, indices);
}

// R-MAT graph on 2^scale x 2^scale with quadrant probabilities a,b,c (d = 1-a-b-c).
// Destination = row.  With halo_log2 >= 0 the matrix models one partition's share: n_dst =
// 2^scale owned rows, n_src = 2^scale + 2^halo_log2; a draw points into the halo with
// probability halo_prob (source = 2^scale + (col >> (scale - halo_log2))).  Node ids are
// scrambled by seeded bijections (separately inside the owned and the halo range).
// One self-loop per owned node.  indices must have room for draws + 2^scale entries.
int64_t gen_rmat(int scale, int64_t draws, double a, double b, double c, int halo_log2,
                 double halo_prob, uint64_t seed, int64_t* indptr, int32_t* indices) {
    const int64_t n = (int64_t)1 << scale;
    std::vector<int32_t> perm_owned, perm_halo;
    make_permutation(perm_owned, n, seed, 6);
    if (halo_log2 >= 0) make_permutation(perm_halo, (int64_t)1 << halo_log2, seed, 7);
    std::vector<int32_t> dst((size_t)(draws + n)), src((size_t)(draws + n));
    const double ab = a + b, abc = a + b + c;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < draws; ++t) {
        int64_t r = 0, col = 0;
        for (int lv = 0; lv < scale; ++lv) {
            double u = rnd_unit(seed, 0, (uint64_t)t * 64u + (uint64_t)lv);
            int rb = u >= ab;                       // quadrants c,d -> lower half (row bit 1)
            int cb = (u >= a && u < ab) || u >= abc;  // quadrants b,d -> right half (col bit 1)
            r = (r << 1) | rb;
            col = (col << 1) | cb;
        }
        int32_t d = perm_owned[(size_t)r];
        int32_t s;
        if (halo_log2 >= 0 && rnd_unit(seed, 1, (uint64_t)t) < halo_prob)
            s = (int32_t)(n + perm_halo[(size_t)(col >> (scale - halo_log2))]);
        else
            s = perm_owned[(size_t)col];
        dst[(size_t)t] = d;
        src[(size_t)t] = s;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        dst[(size_t)(draws + i)] = (int32_t)i;
        src[(size_t)(draws + i)] = (int32_t)i;
    }
    return build_csr(dst, src, n, indptr, indices);
}

// n independent N(0,1) samples (Box-Muller on counter-based uniforms), fp32.
void gen_normal_f32(float* out, int64_t n, uint64_t seed, uint64_t stream) {
    const int64_t pairs = (n + 1) / 2;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < pairs; ++p) {
        double u1 = rnd_unit(seed, stream, (uint64_t)(2 * p));
        double u2 = rnd_unit(seed, stream, (uint64_t)(2 * p + 1));
        double rad = std::sqrt(-2.0 * std::log(u1));
        double ang = 6.283185307179586476925 * u2;
        out[2 * p] = (float)(rad * std::cos(ang));
        if (2 * p + 1 < n) out[2 * p + 1] = (float)(rad * std::sin(ang));
    }
}

// Same samples rounded to bfloat16 (round to nearest even), returned as raw 16-bit patterns.
void gen_normal_bf16(uint16_t* out, int64_t n, uint64_t seed, uint64_t stream) {
    const int64_t pairs = (n + 1) / 2;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < pairs; ++p) {
        double u1 = rnd_unit(seed, stream, (uint64_t)(2 * p));
        double u2 = rnd_unit(seed, stream, (uint64_t)(2 * p + 1));
        double rad = std::sqrt(-2.0 * std::log(u1));
        double ang = 6.283185307179586476925 * u2;
        out[2 * p] = f32_to_bf16_rne((float)(rad * std::cos(ang)));
        if (2 * p + 1 < n) out[2 * p + 1] = f32_to_bf16_rne((float)(rad * std::sin(ang)));
    }
}

}  // extern "C"
