/* gta — sparse graph attention for one MI355X (gfx950): C ABI.
 *
 * The library computes the attention core of a sparse graph transformer layer (paper Section
 * 2.1, Eq. 2, 4, 5; multi-head form as described after Eq. 5) and its gradients (Section 2.2)
 * for one GPU's share of the graph:
 *
 *     s[e,h]   = scale * sum_d Q[i,h,d] * K[j,h,d]        for every stored entry e = (i <- j)   (SDDMM)
 *     a[e,h]   = exp(s[e,h]) / sum_{e' in row i} exp(s[e',h])                                  (edge softmax)
 *     out[i,h] = sum_{e in row i} a[e,h] * V[j,h,:]                                            (SpMM)
 *
 * The graph is CSR by destination: row i of `indptr`/`indices` lists the sources j that node i
 * attends to.  Rows are the n_dst nodes owned by this GPU; sources are n_src >= n_dst rows of
 * K/V (owned nodes first, then halo rows gathered from other GPUs, Algorithm 1).  Every stored
 * entry is one softmax term (repeated entries count repeatedly, rows need not be sorted).  A row
 * without entries yields out = 0, lse = -inf and no gradient.
 *
 * Pointers.  Unless a parameter says "host", every pointer is a DEVICE pointer owned by the
 * caller, valid on the current HIP device until the stream work queued by the call has finished.
 * The library allocates no device memory: plan storage and per-call scratch are caller-provided
 * (sizes come from the *_bytes queries).  `stream` is a hipStream_t passed as void* (NULL = the
 * default stream).  gta_attn_fwd / gta_attn_bwd only enqueue work; gta_plan_create synchronises
 * the stream before returning.
 *
 * Layout.  Q, out, dOut, dQ: [n_dst, heads, head_dim]; K, V, dK, dV: [n_src, heads, head_dim];
 * row-major, contiguous, base 16-byte aligned; elements float (GTA_F32) or bfloat16 (GTA_BF16).
 * lse: float [n_dst, heads], natural-log sum of exp of the scaled scores.  Accumulation is
 * always fp32; bf16 outputs are rounded to nearest even.
 *
 * Supported shapes: head_dim * sizeof(element) in {16, 32, 64, 128, 256} bytes; n_dst, n_src
 * < 2^31, nnz <= 2^31 - 1024.  A row is processed slice_heads heads at a time, slice_heads being the largest power
 * of two that divides `heads` and keeps a slice within 1024 bytes; a slice must span at least
 * 64 bytes.  Power-of-two head counts with rows up to 1024 bytes run in one launch per pass (the
 * tuned case); wider rows and other head counts take one launch per slice.
 *
 * Errors.  Every call returns a gta_status and never aborts; on error no output is defined.
 * gta_last_error() gives a thread-local message for the last failing call of this thread.
 */
#ifndef GTA_H_
#define GTA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GTA_OK = 0,
    GTA_ERR_INVALID_ARG = 1, /* null pointer, negative size, misaligned base, inconsistent sizes */
    GTA_ERR_UNSUPPORTED = 2, /* shape or dtype outside the supported set                        */
    GTA_ERR_WORKSPACE = 3,   /* workspace / scratch buffer too small                            */
    GTA_ERR_HIP = 4,         /* a HIP runtime call failed (message in gta_last_error)           */
    GTA_ERR_GRAPH = 5        /* validate=1 found a malformed CSR                                */
} gta_status;

typedef enum { GTA_F32 = 0, GTA_BF16 = 1 } gta_dtype;

typedef struct gta_plan gta_plan; /* opaque, host-side handle */

/* Scheduling thresholds; 0 selects the default (wave_max_deg 128, hub_chunk 2048).  wave_max_deg and
 * hub_chunk must be powers of two with hub_chunk >= wave_max_deg.
 *   rows with degree <= wave_max_deg  : one wavefront (or a fraction of one) per row
 *   rows with degree  > wave_max_deg  : cut into chunks of hub_chunk entries, one workgroup per
 *                                       chunk; rows with more than one chunk are merged afterwards
 *   pack_max_deg                      : rows up to this degree are packed several to a wavefront
 *                                       (0 = chosen per shape at launch)
 *   validate                          : 1 = check indptr / indices at plan creation
 *   keep_dz_min_nnz                   : the backward keeps dZ per stored entry (needs the recommended
 *                                       scratch size) only for graphs with at least this many entries;
 *                                       0 = default (262144: below that the extra launch costs more
 *                                       than the saved gathers), 1 = always, negative = never          */
typedef struct {
    int32_t pack_max_deg;
    int32_t wave_max_deg;
    int32_t hub_chunk;
    int32_t validate;
    int32_t keep_dz_min_nnz;
} gta_plan_opts;

#define GTA_NUM_CLASSES 33 /* degree classes: 0 for degree 0, else 1 + ceil(log2(degree)) */

typedef struct {
    int64_t n_dst, n_src, nnz;
    int32_t pack_max_deg, wave_max_deg, hub_chunk;
    /* per side (0 = destination rows / in-degree, 1 = source rows / out-degree):              */
    int64_t n_chunked[2]; /* rows with degree > wave_max_deg (a prefix of bin_rows)             */
    int64_t n_hub[2];     /* rows with degree > hub_chunk    (a prefix of bin_rows)             */
    int64_t n_chunks[2];  /* entries of the chunk table                                         */
} gta_plan_info;

/* Bytes of device workspace gta_plan_create needs for a graph of this size (0 on bad args). */
size_t gta_plan_workspace_bytes(int64_t n_dst, int64_t n_src, int64_t nnz, const gta_plan_opts* opts);

/* Builds the scheduling plan (integer-only; once per graph).  It consists of
 *   - per side, row ids ordered by (degree class descending, row id ascending) with class
 *     offsets, and the chunk table of the rows above wave_max_deg;
 *   - the transposed pattern t_indptr / t_indices / t_eid ordered by (source ascending, stored
 *     position ascending), which fixes the summation order of dK and dV (Section 2.2: dK and dV
 *     are SpMMs with the transposed adjacency).
 * `workspace` must stay allocated, and indptr / indices unchanged, while the plan is in use.
 * *plan is a host object released with gta_plan_destroy (which does not touch the workspace). */
gta_status gta_plan_create(gta_plan** plan, const int64_t* indptr, const int32_t* indices,
                           int64_t n_dst, int64_t n_src, int64_t nnz, const gta_plan_opts* opts,
                           void* workspace, size_t workspace_bytes, void* stream);
void gta_plan_destroy(gta_plan* plan);

/* Only the leading gta_plan_retained_bytes of the workspace stay in use once gta_plan_create has
 * returned (the rest held sort buffers).  gta_plan_compact copies that part into new_workspace
 * (device, 256-byte aligned, at least gta_plan_retained_bytes, not overlapping it) and makes the plan
 * use the copy, after which the caller may release the original buffer: on the largest benchmark
 * workload that leaves 0.9 GB instead of 1.9 GB beside the tensors.  Synchronises the stream; no
 * other call may be using the plan meanwhile. */
size_t gta_plan_retained_bytes(int64_t n_dst, int64_t n_src, int64_t nnz, const gta_plan_opts* opts);
gta_status gta_plan_compact(gta_plan* plan, void* new_workspace, size_t new_workspace_bytes, void* stream);

gta_status gta_plan_get_info(const gta_plan* plan, gta_plan_info* info /* host */);

/* Copies plan arrays to HOST buffers (any may be NULL to skip); synchronises the device.
 * side 0: destination rows, side 1: source rows.
 *   bin_rows  int32 [n_rows]           bin_off   int64 [GTA_NUM_CLASSES + 1]
 *   chunk_ptr int32 [n_chunked + 1]    chunks    int32 [n_chunks][4] = (row, begin, end, chunks of row) */
gta_status gta_plan_export_bins(const gta_plan* plan, int side, int32_t* bin_rows, int64_t* bin_off,
                                int32_t* chunk_ptr, int32_t* chunks);
/* t_indptr int64 [n_src + 1], t_indices int32 [nnz] (destination of each transposed entry),
 * t_eid int32 [nnz] (its position in `indices`); HOST buffers, any may be NULL. */
gta_status gta_plan_export_transpose(const gta_plan* plan, int64_t* t_indptr, int32_t* t_indices,
                                     int32_t* t_eid);

/* Bytes of device scratch for gta_attn_fwd / gta_attn_bwd (0 on bad args).
 * gta_attn_scratch_bytes     : recommended size.  Besides the partial results of split rows and the
 *                              per-row statistics it holds dZ as float [nnz, heads], which lets the
 *                              backward gather three rows per entry instead of four.
 * gta_attn_scratch_bytes_min : smallest size accepted.  With less than the recommended size the
 *                              backward keeps nothing per entry and recomputes dZ in both of its
 *                              passes (same results up to rounding, about 20 % slower).
 * For rows (head slices) of up to 128 bytes the two sizes are equal: there the recomputing form is
 * the faster one and is always used.                                                              */
size_t gta_attn_scratch_bytes(const gta_plan* plan, int heads, int head_dim, gta_dtype dtype);
size_t gta_attn_scratch_bytes_min(const gta_plan* plan, int heads, int head_dim, gta_dtype dtype);

/* Forward (Eq. 4-5 fused: SDDMM -> edge softmax -> SpMM, scores never stored).
 * scale <= 0 selects 1/sqrt(head_dim).  Writes every row of out and lse. */
gta_status gta_attn_fwd(const gta_plan* plan, const int64_t* indptr, const int32_t* indices,
                        const void* Q, const void* K, const void* V, void* out, float* lse,
                        int64_t n_dst, int64_t n_src, int heads, int head_dim, gta_dtype dtype,
                        float scale, void* scratch, size_t scratch_bytes, void* stream);

/* Backward (Section 2.2: dV = U^T dY, dU = SDDMM(A, dY, V^T), softmax backward, dQ = dZ K,
 * dK = dZ^T Q), with the weights recomputed from lse instead of stored.  out and lse are the
 * forward results.  Writes every row of dQ, dK and dV (dK/dV for all n_src rows, zero where a
 * source has no entry).  Bitwise reproducible: no floating-point atomics, fixed summation order. */
gta_status gta_attn_bwd(const gta_plan* plan, const int64_t* indptr, const int32_t* indices,
                        const void* Q, const void* K, const void* V, const void* out,
                        const float* lse, const void* dOut, void* dQ, void* dK, void* dV,
                        int64_t n_dst, int64_t n_src, int heads, int head_dim, gta_dtype dtype,
                        float scale, void* scratch, size_t scratch_bytes, void* stream);

/* gta_attn_fwd for callers that cannot allocate device memory and have no scratch buffer to pass:
 * code running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * call allocates nothing: the partial results of the rows cut into several chunks (degree >
 * hub_chunk) go to a fixed GTA_NOALLOC_SCRATCH_BYTES array inside the library's device image, which
 * every GPU the library runs on holds until the process ends.  The first call on a device looks the
 * array's device address up once (hipGetSymbolAddress, with that device current) and keeps it; make
 * that call outside a graph capture.  Launch timing (gta_profile_enable) creates events and must be
 * off for such callers.
 * A graph whose split rows need more (chunks of such rows x heads x (head_dim + 2 values per
 * 16 bytes of a head) x 4 bytes) is rejected with GTA_ERR_WORKSPACE; use gta_attn_fwd then.
 * All calls on one GPU share that array: calls that overlap on one GPU (two streams, two threads)
 * race on it; calls on one stream, or otherwise ordered, do not.  Nothing in it needs clearing
 * between calls: every value read was written earlier by the same call.  Inputs, outputs, results
 * (bitwise) and all other rules are those of gta_attn_fwd. */
#define GTA_NOALLOC_SCRATCH_BYTES ((size_t)16 << 20)
gta_status gta_attn_fwd_noalloc(const gta_plan* plan, const int64_t* indptr, const int32_t* indices,
                                const void* Q, const void* K, const void* V, void* out, float* lse,
                                int64_t n_dst, int64_t n_src, int heads, int head_dim, gta_dtype dtype,
                                float scale, void* stream);

/* The same two calls for a GPU whose K / V rows sit in two allocations (Section 3.1, Algorithm 1:
 * the rows it owns, and the halo rows an all-gather delivered into a receive buffer), so that no
 * concatenated copy has to be made.  Source ids 0 .. n_local-1 address K_local / V_local
 * [n_local, heads, head_dim], ids n_local .. n_src-1 address row (id - n_local) of K_halo / V_halo
 * [n_src - n_local, heads, head_dim]; the backward writes dK / dV the same way (the halo part is
 * what a reduce-scatter returns to the owners).  0 <= n_local <= n_src; the halo pointers may be
 * NULL only when n_local == n_src.  Results are bitwise those of gta_attn_fwd / gta_attn_bwd on
 * the concatenated tensors.  Everything else as above. */
gta_status gta_attn_fwd_halo(const gta_plan* plan, const int64_t* indptr, const int32_t* indices,
                             const void* Q, const void* K_local, const void* V_local,
                             const void* K_halo, const void* V_halo, int64_t n_local, void* out,
                             float* lse, int64_t n_dst, int64_t n_src, int heads, int head_dim,
                             gta_dtype dtype, float scale, void* scratch, size_t scratch_bytes,
                             void* stream);
gta_status gta_attn_bwd_halo(const gta_plan* plan, const int64_t* indptr, const int32_t* indices,
                             const void* Q, const void* K_local, const void* V_local,
                             const void* K_halo, const void* V_halo, int64_t n_local, const void* out,
                             const float* lse, const void* dOut, void* dQ, void* dK_local,
                             void* dV_local, void* dK_halo, void* dV_halo, int64_t n_dst, int64_t n_src,
                             int heads, int head_dim, gta_dtype dtype, float scale, void* scratch,
                             size_t scratch_bytes, void* stream);

/* Combines two forward results computed over DISJOINT sets of stored entries of the same rows
 * (two plans over the same n_rows destinations, e.g. the entries whose sources are owned rows and
 * the entries whose sources are halo rows of Algorithm 1, so that the first can run before the halo
 * has arrived): per row and head, lse = log(exp(lse_a) + exp(lse_b)) and
 * out = exp(lse_a - lse) out_a + exp(lse_b - lse) out_b, which is Eq. 2 over the union.  A side with
 * lse = -inf contributes nothing.  out may alias out_a or out_b; lse must not alias lse_a / lse_b.
 * The merged out and lse are what gta_attn_bwd expects when it is then called once per entry set
 * (same Q, out, lse, dOut): the two dQ results add, dK / dV add where a source is in both sets. */
gta_status gta_attn_merge(const void* out_a, const float* lse_a, const void* out_b, const float* lse_b,
                          void* out, float* lse, int64_t n_rows, int heads, int head_dim,
                          gta_dtype dtype, void* stream);

/* ---- The same computation as separate operators (Section 2.2 counts them: forward = 1 SDDMM +
 * softmax + 1 SpMM, backward = 3 SpMM + 1 SDDMM), with the per-entry matrices stored as
 * float [nnz, heads] in the order of `indices`.  Not used by gta_attn_fwd/bwd; provided so the
 * unfused decomposition can be run and timed operator by operator.  scratch: as for gta_attn_fwd.
 *
 * gta_sddmm:            Z[e,h]  = sum_d X[i,h,d] * Y[j,h,d]          X [n_dst,H,D], Y [n_src,H,D]
 * gta_edge_softmax:     U[e,h]  = softmax over row i of scale*Z[.,h]; lse (may be NULL) [n_dst,H]
 * gta_edge_softmax_bwd: dZ[e,h] = scale * U[e,h] * (dU[e,h] - sum_{e' in row i} U[e',h] dU[e',h])
 * gta_spmm:   transposed = 0:  Y[i,h,:] = sum_{e=(i<-j)} W[e,h] * X[j,h,:]   X [n_src,..], Y [n_dst,..]
 *             transposed = 1:  Y[j,h,:] = sum_{e=(i<-j)} W[e,h] * X[i,h,:]   X [n_dst,..], Y [n_src,..]
 *             (terms of a row are added in the plan's fixed order; no atomics)                      */
gta_status gta_sddmm(const gta_plan* plan, const int64_t* indptr, const int32_t* indices, const void* X,
                     const void* Y, float* Z, int64_t n_dst, int64_t n_src, int heads, int head_dim,
                     gta_dtype dtype, void* scratch, size_t scratch_bytes, void* stream);
gta_status gta_edge_softmax(const gta_plan* plan, const int64_t* indptr, const float* Z, float* U,
                            float* lse, int64_t n_dst, int heads, float scale, void* stream);
gta_status gta_edge_softmax_bwd(const gta_plan* plan, const int64_t* indptr, const float* U,
                                const float* dU, float* dZ, int64_t n_dst, int heads, float scale,
                                void* stream);
gta_status gta_spmm(const gta_plan* plan, const int64_t* indptr, const int32_t* indices, const float* W,
                    const void* X, void* Y, int64_t n_dst, int64_t n_src, int heads, int head_dim,
                    gta_dtype dtype, int transposed, void* scratch, size_t scratch_bytes, void* stream);

/* ---- Dense projections of the layer on the matrix cores (Eq. 3: Q,K,V = X W_Q, X W_K, X W_V;
 * Eq. 5: X' = X W_o + Y) and their gradients.  bfloat16 or fp32 operands (all tensors of a call in
 * the same type), fp32 accumulation; row-major, contiguous, 16-byte aligned.  d_in (the reduction
 * length) must be a multiple of 16 and at most 512 (bfloat16) / 496 (fp32) for gta_linear, d_out a
 * multiple of 8.
 * gta_linear:    Y[n, d_out] = X[n, d_in] * op(W) (+ C)      C [n, d_out] may be NULL, and may be Y
 *                itself (in-place accumulation: every element of C is read before it is written)
 *                trans_w = 0: W is [d_in, d_out] (Y = X W);   trans_w = 1: W is [d_out, d_in] (Y = X W^T,
 *                the form of dX = dY W^T).
 * gta_linear_dw: dW[d_in, d_out] (float) = X^T dY, X [n, d_in], dY [n, d_out]; row blocks are summed
 *                in a fixed order (no atomics).  scratch: gta_linear_dw_scratch_bytes.             */
gta_status gta_linear(const void* X, const void* W, const void* C, void* Y, int64_t n, int d_in, int d_out,
                      gta_dtype dtype, int trans_w, void* stream);
size_t gta_linear_dw_scratch_bytes(int64_t n, int d_in, int d_out);
gta_status gta_linear_dw(const void* X, const void* dY, float* dW, int64_t n, int d_in, int d_out,
                         gta_dtype dtype, void* scratch, size_t scratch_bytes, void* stream);

/* p weight gradients of one shape (1 <= p <= 4), dW[k] = X[k]^T dY[k], each exactly what gta_linear_dw
 * gives (same blocks, same summation order).  bfloat16: one launch; products that name the same X (the
 * gradients of W_Q, W_K, W_V, W_o in Eq. 3 and 5 all multiply the layer input) run side by side on one
 * XCD, so the X rows one of them fetches serve the others from that L2.  float: one product after the
 * other.  X, dY, dW are HOST arrays of p device pointers; the dW[k] must be distinct.
 * scratch (device): gta_linear_dw_group_scratch_bytes = p x gta_linear_dw_scratch_bytes.               */
size_t gta_linear_dw_group_scratch_bytes(int64_t n, int d_in, int d_out, int p);
gta_status gta_linear_dw_group(const void* const* X, const void* const* dY, float* const* dW, int p, int64_t n,
                               int d_in, int d_out, gta_dtype dtype, void* scratch, size_t scratch_bytes,
                               void* stream);

/* Several projections that share operands, in one launch (bfloat16, d in {64, 128, 256}):
 *     Y[po][n, d] = sum_{pi < p_in} X[pi][n, d] * op(W[po * p_in + pi]) (+ C[po])      for po < p_out
 * with op as in gta_linear (trans_w = 0: W is [d, d] input x output; 1: output x input), fp32
 * accumulation over all p_in products and ONE rounding.  Every X[pi] is read from memory once, also
 * when several outputs use it, and every Y[po] is written once.  Supported groupings: (p_in, p_out) =
 * (1, 1) with or without addends, (1, 3) (Eq. 3: Q, K, V from one read of X) and (4, 1) (the input
 * gradient dX = dX' W_o^T + dQ W_Q^T + dK W_K^T + dV W_V^T) without.  X, W, C (NULL, or p_out
 * non-null addends), Y are HOST arrays of device pointers; no output may alias an input or addend.
 * scratch (device, 256-byte aligned): gta_linear_group_scratch_bytes, used for the repacked weights. */
size_t gta_linear_group_scratch_bytes(int d, int p_in, int p_out);
gta_status gta_linear_group(const void* const* X, int p_in, const void* const* W, int p_out,
                            const void* const* C, void* const* Y, int64_t n, int d, gta_dtype dtype,
                            int trans_w, void* scratch, size_t scratch_bytes, void* stream);

/* ---- One Sparse Graph Attention layer (Eq. 3-5) on one GPU with n_src == n_dst == n, bfloat16 or fp32:
 *   Q,K,V = X W_Q, X W_K, X W_V;   Y = attention(Q,K,V);   X' = X W_o + Y.
 * X, Q, K, V, Y, X' are [n, d] = [n, heads, head_dim]; weights are [d, d] (input x output).
 * Forward writes Q, K, V, Y, lse (kept for the backward) and Xout.  Backward takes dXout and writes
 * dX [n, d], the weight gradients dW_* (float [d, d]) and uses dQ, dK, dV [n, d] as work buffers.
 * bfloat16 layers with d in {64, 128, 256} compute Q, K, V in one launch (X read once) and dX as one
 * four-term sum in fp32, rounded once (gta_linear_group); other shapes run one product per launch
 * and accumulate dX through the tensor type (rounded after each).  The four weight gradients, which all
 * multiply X, go through gta_linear_dw_group.  scratch:
 * gta_sga_layer_scratch_bytes.  Host-side sequencing of the entry points above.                  */
size_t gta_sga_layer_scratch_bytes(const gta_plan* plan, int heads, int head_dim, gta_dtype dtype);
gta_status gta_sga_layer_fwd(const gta_plan* plan, const int64_t* indptr, const int32_t* indices,
                             const void* X, const void* Wq, const void* Wk, const void* Wv, const void* Wo,
                             void* Q, void* K, void* V, void* Y, float* lse, void* Xout, int64_t n,
                             int heads, int head_dim, gta_dtype dtype, float scale, void* scratch,
                             size_t scratch_bytes, void* stream);
gta_status gta_sga_layer_bwd(const gta_plan* plan, const int64_t* indptr, const int32_t* indices,
                             const void* X, const void* Wq, const void* Wk, const void* Wv, const void* Wo,
                             const void* Q, const void* K, const void* V, const void* Y, const float* lse,
                             const void* dXout, void* dQ, void* dK, void* dV, void* dX, float* dWq,
                             float* dWk, float* dWv, float* dWo, int64_t n, int heads, int head_dim,
                             gta_dtype dtype, float scale, void* scratch, size_t scratch_bytes, void* stream);

/* ---- Layout transforms of GP-A2A (Section 3.2, Algorithm 2: [(N/p),h,d'] <-> [N,(h/p),d']).
 * gta_head_split regroups X [n_rows, heads, head_dim] into `parts` contiguous blocks
 * S [parts][n_rows, heads/parts, head_dim] (block r is what GPU r receives from this GPU);
 * gta_head_merge is the inverse.  heads must be divisible by parts and a head block must be a
 * multiple of 16 bytes.  The exchange itself (an all-to-all) is not part of this library.       */
gta_status gta_head_split(const void* X, void* S, int64_t n_rows, int heads, int head_dim,
                          gta_dtype dtype, int parts, void* stream);
gta_status gta_head_merge(const void* S, void* X, int64_t n_rows, int heads, int head_dim,
                          gta_dtype dtype, int parts, void* stream);

/* ---- Automatic Graph Parallelism (Section 4.3, Algorithm 3).  Host arithmetic only; all pointers
 * are HOST pointers.  With k = t_iter(1) / N, every measured coefficient beta_c(i) (seconds per
 * node for strategy c on i GPUs, 2 <= i <= max_gpus) gives the term i * beta / (i - 1); the entry
 * with the smallest term that does not exceed k is selected (ties: fewer GPUs, then first in table order).
 * *strategy = its strategy id and *gpus = i, or (-1, 1) when no entry qualifies (stay on one
 * GPU).  est_t_iter (may be NULL) receives t_iter(1)/i + beta * N for the selection (Eq. 7 with
 * alpha(i) = alpha(1)/i).  This build runs on one GPU, so the coefficients must come from elsewhere. */
typedef struct {
    int32_t strategy; /* caller-defined id, e.g. 0 = GP-AG, 1 = GP-A2A */
    int32_t gpus;     /* i                                              */
    double beta;      /* beta_c(i), seconds per node                    */
} gta_agp_sample;
gta_status gta_agp_select(double t_iter1_seconds, int64_t n_nodes, const gta_agp_sample* samples,
                          int n_samples, int max_gpus, int* strategy, int* gpus, double* est_t_iter);

/* Per-launch timing for benchmarks.  While enabled (on = 1), every kernel launch of
 * gta_attn_fwd/bwd is bracketed by HIP events on the call's stream.  on = 2 additionally launches
 * the three row schedules of a pass separately (instead of in one grid) so each is timed alone.  gta_profile_read synchronises those events and
 * copies up to `cap` records to HOST memory (oldest first), returns how many launches were
 * recorded since the last reset, and clears the list when reset != 0. */
typedef struct {
    char name[40];   /* "fwd", "bwd_dst", "bwd_src" (+ ".merge"; with on = 2: ".chunk", ".wave", ".packed") */
    float ms;        /* elapsed time of this launch     */
    int64_t rows;    /* rows it processed               */
    int64_t entries; /* stored entries it processed     */
} gta_launch_record;
gta_status gta_profile_enable(int on);
int gta_profile_read(gta_launch_record* out, int cap, int reset);

/* Streaming probe for benchmarks: one plain kernel over `bytes` bytes (a multiple of 16) per operand,
 * so that the attention passes can be read against the bandwidth a streaming kernel reaches on the
 * same GPU in the same run.  mode 0: reads a (dst needs 16 writable bytes; they are written only if the
 * XOR of everything a thread read equals one chosen 32-bit pattern, which is what keeps the reads alive);
 * mode 1: dst = a; mode 2: dst = a + b as floats.  Timed like every other launch while
 * gta_profile_enable is on (records "probe_read" / "probe_copy" / "probe_add", entries = bytes / 16). */
gta_status gta_stream_probe(int mode, void* dst, const void* a, const void* b, size_t bytes, void* stream);

const char* gta_last_error(void);
const char* gta_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GTA_H_ */
