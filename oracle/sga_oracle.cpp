// CPU oracle for sparse graph attention (SGA): TEST INFRASTRUCTURE ONLY.
//
// Only tests, the smoke check and the benchmark's cpu_baseline leg may call this file.  It
// shares no code with the GPU library and is never a fallback for it.
//
// It is the paper's definition written out, one function per operator, in double precision,
// with no blocking, fusion or reordering:
//   forward  (Section 2.1, Eq. 3-5; multi-head as described after Eq. 5):
//       Z = (Q K^T) (.) A          -> sga_sddmm           (one value per stored entry and head)
//       U = Softmax(Z / sqrt(d))   -> sga_edge_softmax    (over the stored entries of a row)
//       Y = U V                    -> sga_spmm
//   backward (Section 2.2: the SpMM needs one SpMM and one SDDMM, the SDDMM needs two SpMM):
//       dV = U^T dY                -> sga_spmm_t          (SpMM with the transposed pattern)
//       dU = (dY V^T) (.) A        -> sga_sddmm
//       dZ = softmax backward      -> sga_edge_softmax_bwd
//       dQ = dZ K                  -> sga_spmm
//       dK = dZ^T Q                -> sga_spmm_t
//
// Conventions.  A is CSR by destination: row i of A lists the sources j in N(i), i.e.
// indices[indptr[i] .. indptr[i+1]).  Every stored entry is one softmax term (a repeated
// entry counts twice).  Dense tensors are row-major [rows, H, D]; per-edge tensors are [E, H].
// The scale 1/sqrt(d) is passed in by the caller.  A row with no entries yields Y = 0 and
// lse = -infinity and contributes to no gradient.
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <vector>

extern "C" {

// Z[e,h] = sum_d X[i,h,d] * Y[j,h,d] for every stored entry e = (i <- j).        (Eq. 4, left)
void sga_sddmm(int64_t n_dst, const int64_t* indptr, const int32_t* indices, int H, int D,
               const double* X, const double* Y, double* Z) {
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = 0; i < n_dst; ++i)
        for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e) {
            const int64_t j = indices[e];
            for (int h = 0; h < H; ++h) {
                double acc = 0.0;
                for (int d = 0; d < D; ++d) acc += X[(i * H + h) * D + d] * Y[(j * H + h) * D + d];
                Z[e * H + h] = acc;
            }
        }
}

// U[e,h] = exp(scale*Z[e,h]) / sum_{e' in row} exp(scale*Z[e',h]);  lse = log of that sum.
// Evaluated with the row maximum subtracted.                                   (Eq. 2, Eq. 4, right)
void sga_edge_softmax(int64_t n_dst, const int64_t* indptr, int H, double scale, const double* Z,
                      double* U, double* lse) {
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = 0; i < n_dst; ++i)
        for (int h = 0; h < H; ++h) {
            const int64_t b = indptr[i], t = indptr[i + 1];
            if (b == t) {
                lse[i * H + h] = -std::numeric_limits<double>::infinity();
                continue;
            }
            double m = scale * Z[b * H + h];
            for (int64_t e = b; e < t; ++e) m = std::fmax(m, scale * Z[e * H + h]);
            double sum = 0.0;
            for (int64_t e = b; e < t; ++e) sum += std::exp(scale * Z[e * H + h] - m);
            for (int64_t e = b; e < t; ++e) U[e * H + h] = std::exp(scale * Z[e * H + h] - m) / sum;
            lse[i * H + h] = m + std::log(sum);
        }
}

// Y[i,h,:] = sum_{e=(i<-j)} W[e,h] * X[j,h,:]                                        (Eq. 5, left)
void sga_spmm(int64_t n_dst, const int64_t* indptr, const int32_t* indices, int H, int D,
              const double* W, const double* X, double* Y) {
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = 0; i < n_dst; ++i) {
        for (int k = 0; k < H * D; ++k) Y[i * H * D + k] = 0.0;
        for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e) {
            const int64_t j = indices[e];
            for (int h = 0; h < H; ++h)
                for (int d = 0; d < D; ++d)
                    Y[(i * H + h) * D + d] += W[e * H + h] * X[(j * H + h) * D + d];
        }
    }
}

// SpMM with the transposed pattern: Y[j,h,:] = sum_{e=(i<-j)} W[e,h] * X[i,h,:], written as
// the scatter it is, in stored order (serial, so the order is the definition's).
void sga_spmm_t(int64_t n_dst, int64_t n_src, const int64_t* indptr, const int32_t* indices, int H,
                int D, const double* W, const double* X, double* Y) {
    for (int64_t k = 0; k < n_src * H * D; ++k) Y[k] = 0.0;
    for (int64_t i = 0; i < n_dst; ++i)
        for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e) {
            const int64_t j = indices[e];
            for (int h = 0; h < H; ++h)
                for (int d = 0; d < D; ++d)
                    Y[(j * H + h) * D + d] += W[e * H + h] * X[(i * H + h) * D + d];
        }
}

// Same result as sga_spmm_t, arranged so rows of Y can be computed in parallel: the entries
// are first grouped by source (stable, so each Y row still adds its terms in stored order).
void sga_spmm_t_grouped(int64_t n_dst, int64_t n_src, const int64_t* indptr, const int32_t* indices,
                        int H, int D, const double* W, const double* X, double* Y) {
    const int64_t nnz = indptr[n_dst];
    std::vector<int64_t> start((size_t)n_src + 1, 0);
    for (int64_t e = 0; e < nnz; ++e) start[(size_t)indices[e] + 1]++;
    for (int64_t j = 0; j < n_src; ++j) start[(size_t)j + 1] += start[(size_t)j];
    std::vector<int64_t> eid((size_t)nnz), row((size_t)nnz);
    {
        std::vector<int64_t> cur(start.begin(), start.end() - 1);
        for (int64_t i = 0; i < n_dst; ++i)
            for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e) {
                const int64_t p = cur[(size_t)indices[e]]++;
                eid[(size_t)p] = e;
                row[(size_t)p] = i;
            }
    }
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t j = 0; j < n_src; ++j) {
        for (int k = 0; k < H * D; ++k) Y[j * H * D + k] = 0.0;
        for (int64_t p = start[(size_t)j]; p < start[(size_t)j + 1]; ++p) {
            const int64_t e = eid[(size_t)p], i = row[(size_t)p];
            for (int h = 0; h < H; ++h)
                for (int d = 0; d < D; ++d)
                    Y[(j * H + h) * D + d] += W[e * H + h] * X[(i * H + h) * D + d];
        }
    }
}

// Derivative of U = softmax(scale*Z) over each row's stored entries:
// dZ[e,h] = scale * U[e,h] * (dU[e,h] - sum_{e' in row} U[e',h] dU[e',h]).
void sga_edge_softmax_bwd(int64_t n_dst, const int64_t* indptr, int H, double scale,
                          const double* U, const double* dU, double* dZ) {
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = 0; i < n_dst; ++i)
        for (int h = 0; h < H; ++h) {
            double dot = 0.0;
            for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e) dot += U[e * H + h] * dU[e * H + h];
            for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e)
                dZ[e * H + h] = scale * U[e * H + h] * (dU[e * H + h] - dot);
        }
}

// Forward of the attention core: Y (and lse; optionally U) from Q, K, V.
int sga_forward(int64_t n_dst, int64_t n_src, const int64_t* indptr, const int32_t* indices, int H,
                int D, double scale, const double* Q, const double* K, const double* V, double* Y,
                double* lse, double* U_out /* may be null */) {
    (void)n_src;
    const int64_t nnz = indptr[n_dst];
    std::vector<double> Z((size_t)nnz * H), U((size_t)nnz * H);
    sga_sddmm(n_dst, indptr, indices, H, D, Q, K, Z.data());
    sga_edge_softmax(n_dst, indptr, H, scale, Z.data(), U.data(), lse);
    sga_spmm(n_dst, indptr, indices, H, D, U.data(), V, Y);
    if (U_out) std::memcpy(U_out, U.data(), sizeof(double) * (size_t)nnz * H);
    return 0;
}

// Gradients of L = sum(dY (.) Y) with respect to Q, K, V.  grouped != 0 uses the grouped
// (parallel) form of the two transposed SpMMs; grouped == 0 the serial scatter.
int sga_backward(int64_t n_dst, int64_t n_src, const int64_t* indptr, const int32_t* indices, int H,
                 int D, double scale, const double* Q, const double* K, const double* V,
                 const double* dY, double* dQ, double* dK, double* dV, int grouped) {
    const int64_t nnz = indptr[n_dst];
    std::vector<double> Z((size_t)nnz * H), U((size_t)nnz * H), dU((size_t)nnz * H),
        dZ((size_t)nnz * H), lse((size_t)n_dst * H);
    sga_sddmm(n_dst, indptr, indices, H, D, Q, K, Z.data());
    sga_edge_softmax(n_dst, indptr, H, scale, Z.data(), U.data(), lse.data());
    auto spmm_t = grouped ? sga_spmm_t_grouped : sga_spmm_t;
    spmm_t(n_dst, n_src, indptr, indices, H, D, U.data(), dY, dV);       // dV = U^T dY
    sga_sddmm(n_dst, indptr, indices, H, D, dY, V, dU.data());           // dU = (dY V^T) (.) A
    sga_edge_softmax_bwd(n_dst, indptr, H, scale, U.data(), dU.data(), dZ.data());
    sga_spmm(n_dst, indptr, indices, H, D, dZ.data(), K, dQ);            // dQ = dZ K
    spmm_t(n_dst, n_src, indptr, indices, H, D, dZ.data(), Q, dK);       // dK = dZ^T Q
    return 0;
}

}  // extern "C"
