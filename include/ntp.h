/*
 * ntp.h - C boundary of the per-worker aggregation hot path of feature-dimension
 * tensor-parallel full-graph GNN training, for one AMD MI355X (gfx950).
 *
 * One worker of the method holds the whole graph and a column slice [N x F_slice] of
 * the vertex features (Section 3.1 of the paper); it aggregates that slice over the
 * normalised adjacency in the forward pass (eq. 1, eq. 3) and over its transpose in the
 * backward pass (Section 4.2.1), optionally chunk by chunk when the topology does not
 * fit the device (Section 4.2.1, Alg. 1), and applies the dense transform of eq. (4).
 *
 * Conventions
 *  - Every call returns an int status: NTP_OK (0) or a negative NTP_E* code.  The text of
 *    the last error on the calling thread is ntp_last_error().
 *  - "host" pointers are ordinary process memory; "device" pointers are HIP device memory
 *    of the current device.  The library never frees or keeps caller buffers: pointers
 *    are used only by the work enqueued during the call.
 *  - Feature / gradient matrices are row-major; ld* are row strides in ELEMENTS (>= the
 *    slice width, < 2^30).  Input and output of one call must not overlap.  Rows are read and
 *    written in aligned vectors of up to 16 bytes; the vector width is the largest that
 *    divides both row strides and the alignment of both base pointers.  When the slice
 *    width is not a multiple of it, the last vector of an input row is read whole, i.e.
 *    up to 15 bytes past the slice but inside the row stride (never written), so padding
 *    the stride of an odd-width slice to a multiple of 4 elements buys the fast path.
 *  - stream arguments are hipStream_t passed as void* (NULL = the null stream).  The
 *    aggregate and nn calls only enqueue work; they do not synchronise with the host.  One
 *    exception: the scratch for the partial sums of split rows is allocated at graph build for
 *    slices of up to 256 columns (and one right-hand side); the first call with a wider slice, or
 *    with more right-hand sides, synchronises the device and allocates a larger one.
 *  - A graph handle may be used by one thread at a time; calls on one handle that overlap
 *    in time on different streams race on its scratch memory.
 */
#ifndef NTP_H
#define NTP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define NTP_OK            0
#define NTP_EINVAL       -1   /* bad argument (null pointer, bad size, id out of range, overlap) */
#define NTP_ENOMEM       -2   /* host or device allocation failed */
#define NTP_EHIP         -3   /* a HIP runtime call failed */
#define NTP_EBUDGET      -4   /* topology not fully device-resident (use the chunked call), or
                                 the device budget cannot hold even the staging buffers */
#define NTP_EUNSUPPORTED -5   /* combination not implemented */

/* ntp_graph_build flags */
#define NTP_SYMMETRISE      1u   /* also add the reverse of every input edge */
#define NTP_DEDUP           2u   /* drop input self loops, keep the first of equal (src,dst) */
#define NTP_ADD_SELF_LOOPS  4u   /* append one (v,v) entry of weight 1 per vertex (A + I) */
#define NTP_NORM_GCN_SYM    8u   /* scale entry (u->v) by 1/sqrt(deg_in(v) * deg_out(u)) */
#define NTP_HOST_ONLY      16u   /* build and plan on the host only; no device memory is
                                    touched; aggregate calls then fail with NTP_EBUDGET */
#define NTP_FORCE_STREAM   32u   /* keep no chunk resident: every chunk is copied from pinned
                                    host memory on every chunked call (cold streaming) */

#define NTP_SCATTER_BWD    64u   /* do not store the by-source form: the backward aggregation
                                    scatter-adds along the by-destination rows with fp32 atomics
                                    (the paper's formulation, Section 4.2.1).  Halves topology
                                    memory and host-link traffic of a directed graph; the order of
                                    the additions, hence the last bits, vary from run to run; fp32
                                    buffers only.  No effect when the adjacency is symmetric. */
#define NTP_EDGE_PERM      128u  /* also keep, for every entry of the by-source form, the position
                                    of the same edge in the by-destination form (4 bytes per entry
                                    on the host and on the device, outside device_budget_bytes;
                                    fewer than 2^31 entries; not with NTP_SCATTER_BWD):
                                    ntp_edge_softmax_bwd then forms every edge's dot product once
                                    instead of once per form */

/* which compressed form */
#define NTP_CSR 0   /* by destination: row v lists in-neighbours u ascending  (forward)  */
#define NTP_CSC 1   /* by source:      row u lists out-neighbours v ascending (backward) */

/* element types of feature / gradient / weight buffers */
#define NTP_F32  0
#define NTP_BF16 1  /* bfloat16 storage, fp32 accumulation, round-to-nearest-even stores */

#define NTP_FWD 0
#define NTP_BWD 1

#define NTP_ACT_NONE 0
#define NTP_ACT_RELU 1

typedef struct ntp_graph ntp_graph_t;

/*
 * Build the normalised adjacency A_hat of Section 4.1.3 (D~^-1/2 (A+I) D~^-1/2 with
 * NTP_SYMMETRISE|NTP_DEDUP|NTP_ADD_SELF_LOOPS|NTP_NORM_GCN_SYM) from a directed edge list
 * and keep it in both compressed forms, as the replicated per-worker topology of
 * Section 3.1.  Edge i is src[i] -> dst[i] (host int32 arrays of n_edges, ids in
 * [0, n_vertices)).  edge_weight (host, nullable) is the per-edge gamma of Section 4.1.3;
 * NULL means 1.  The stored value of an entry is
 *     (float)((double)w * (1.0 / sqrt((double)deg_in(dst) * (double)deg_out(src))))
 * with NTP_NORM_GCN_SYM (degrees = final row lengths, self loop included), else w.
 * Processing order: input order; reversed copies after all originals; dedup keeps the
 * first; self loops last; rows sorted by neighbour id, stable.
 *
 * Chunking (Section 4.2.1): the rows of each form are cut into contiguous ranges of at
 * most chunk_edges entries, greedily, whole rows only; a row with more entries than
 * chunk_edges is cut further by entry range.  chunk_edges = 0 lets the library choose
 * (one chunk if everything fits the budget).  device_budget_bytes bounds the device
 * memory the handle may hold for topology (resident chunks + two staging buffers);
 * 0 = unlimited.  Chunks that fit stay resident from build time on; the others are
 * streamed from pinned host memory by ntp_chunked_aggregate.
 *
 * The input arrays are copied; *out is owned by the library until ntp_graph_free.
 * Errors: NTP_EINVAL (bad ids/sizes/flags), NTP_ENOMEM, NTP_EHIP, NTP_EBUDGET.
 */
int ntp_graph_build(int64_t n_vertices, int64_t n_edges,
                    const int32_t* src, const int32_t* dst, const float* edge_weight,
                    uint32_t flags, int64_t device_budget_bytes, int64_t chunk_edges,
                    ntp_graph_t** out);

/* Sizes of a built graph.  Any out pointer may be NULL.  nnz counts stored entries of the
 * CSR (edges after symmetrisation/dedup + self loops); n_chunks/max_degree refer to the
 * CSR; is_symmetric is 1 when CSC and CSR are bit-identical (the CSC then aliases it). */
int ntp_graph_info(const ntp_graph_t* g, int64_t* n_vertices, int64_t* nnz,
                   int32_t* n_chunks, int32_t* is_symmetric, int64_t* max_degree);

/* Copy one compressed form to host arrays (rowptr[n+1] int64, colidx[nnz] int32,
 * val[nnz] fp32), for bit-exact comparison.  Any of the three may be NULL. */
int ntp_graph_export(const ntp_graph_t* g, int which,
                     int64_t* rowptr, int32_t* colidx, float* val);

/* Copy the edge permutation of a graph built with NTP_EDGE_PERM to perm[nnz] (host int32):
 * perm[k] = position in the by-destination form (ntp_graph_export(NTP_CSR)) of the edge stored at
 * position k of the by-source form.  NTP_EUNSUPPORTED without the flag. */
int ntp_graph_export_perm(const ntp_graph_t* g, int32_t* perm);

/* Chunk table of one form: for chunk c, rows [row_begin[c], row_end[c]) and entries
 * [entry_begin[c], entry_end[c]); resident[c] = 1 if it lives on the device.  Arrays
 * (host, nullable) must hold n_chunks elements; *n_chunks is always written. */
int ntp_graph_chunks(const ntp_graph_t* g, int which, int32_t* n_chunks,
                     int64_t* row_begin, int64_t* row_end,
                     int64_t* entry_begin, int64_t* entry_end, int32_t* resident);

/* Bytes one chunked pass over the form `which` copies from host to device: for every chunk that
 * is not resident its row pointers and row lists plus 4 bytes per entry (column ids), and 4 more
 * (weights) only when the graph was built with caller weights.  Without caller weights the weights
 * of a streamed chunk are rebuilt on the device from the degrees (bit-identical to the stored
 * ones), which halves the host-link traffic of the chunk schedule. */
int ntp_graph_stream_bytes(const ntp_graph_t* g, int which, int64_t* bytes);

/* Device bytes held by the handle (resident topology, staging buffers, scratch). */
int ntp_graph_device_bytes(const ntp_graph_t* g, int64_t* bytes);

/*
 * Forward aggregation of eq. (1)/(3) on one column slice (step 1 of Section 3.1; AGG in
 * Alg. 1):   Y[v, 0:f] = sum over stored entries (v,u) of val(v,u) * X[u, 0:f].
 * X, Y: device, [n_vertices x f_slice] with strides ldx, ldy; dtype NTP_F32 or NTP_BF16.
 * fp32 accumulation; deterministic (no atomics).  Requires a fully resident CSR, else
 * NTP_EBUDGET.  Asynchronous on `stream`.
 */
int ntp_aggregate_fwd(ntp_graph_t* g, const void* X, void* Y,
                      int64_t f_slice, int64_t ldx, int64_t ldy, int dtype, void* stream);

/*
 * ntp_aggregate_fwd for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels
 * and the same bits as ntp_aggregate_fwd, but the partial sums of split rows (rows too long for
 * one wavefront) go to a scratch array that is part of the library image instead of a buffer
 * the handle allocates on first use: the call makes no hipMalloc / hipFree and no
 * synchronisation.  The array holds NTP_NOALLOC_SCRATCH_BYTES on every GPU the library runs on,
 * for the life of the process.  A graph whose split rows need more at this width
 * (pieces of split rows x f_slice rounded up to 8 x 4 bytes) is refused with NTP_EUNSUPPORTED.
 * All calls on one GPU share the array, whatever the handle or stream: calls that overlap in
 * time on one GPU race; nothing in it has to be zero between calls (every slot is written
 * before it is read).
 */
#define NTP_NOALLOC_SCRATCH_BYTES (8ll << 20)
int ntp_aggregate_fwd_noalloc(ntp_graph_t* g, const void* X, void* Y,
                              int64_t f_slice, int64_t ldx, int64_t ldy, int dtype, void* stream);

/*
 * Backward aggregation (Section 4.2.1; AGG of the reverse loop in Alg. 1): the gradient of
 * a source vertex is the weighted sum of the gradients of the vertices it points to,
 *     Gin[u, 0:f] = sum over stored entries (v,u) of val(v,u) * Gout[v, 0:f] = A_hat^T Gout,
 * computed as a gather over the by-source rows.  Same argument rules as the forward.
 */
int ntp_aggregate_bwd(ntp_graph_t* g, const void* Gout, void* Gin,
                      int64_t f_slice, int64_t ldg_out, int64_t ldg_in, int dtype, void* stream);

/*
 * Chunk-scheduled aggregation (Section 4.2.1, inner chunk loop of Alg. 1): same result as
 * ntp_aggregate_fwd / _bwd (direction NTP_FWD / NTP_BWD), produced chunk by chunk.  Against a
 * graph built with another chunking the result agrees to rounding, not in every bit: rows too
 * long for one wavefront are summed in pieces whose length follows the chunk size.  For one
 * graph the result is the same whether a chunk is resident or streamed, and from call to call.
 * Resident chunks are aggregated in place; every other chunk is copied from pinned host
 * memory into one of two device staging buffers on copy_stream while the previous chunk
 * is aggregated on compute_stream (events order the two).  X and Y stay on the device for
 * the whole call.  Works for fully resident graphs too.  On return all work is enqueued;
 * compute_stream has been made to wait for the copies it needs, and the staging buffers
 * are protected across calls by events.  copy_stream must differ from compute_stream
 * when any chunk is streamed (NTP_EINVAL otherwise).
 */
int ntp_chunked_aggregate(ntp_graph_t* g, int direction, const void* X, void* Y,
                          int64_t f_slice, int64_t ldx, int64_t ldy, int dtype,
                          void* compute_stream, void* copy_stream);

/*
 * The same schedule for several right-hand sides (several column slices held by one
 * worker, or the slices of several workers run one after the other on one GPU): every
 * chunk is brought to the device ONCE and applied to all n_rhs inputs before the next
 * chunk is touched, so the host-link traffic of a streamed pass is paid once instead of
 * n_rhs times (the backward sums of Section 4.2.1 stay independent per right-hand side).
 * X and Y are host arrays of n_rhs device pointers (1 <= n_rhs <= 64); all right-hand
 * sides share f_slice, the strides and the dtype; no output may alias any input or other
 * output.  Results are bit-identical to n_rhs separate ntp_chunked_aggregate calls.
 */
int ntp_chunked_aggregate_multi(ntp_graph_t* g, int direction, int32_t n_rhs,
                                const void* const* X, void* const* Y,
                                int64_t f_slice, int64_t ldx, int64_t ldy, int dtype,
                                void* compute_stream, void* copy_stream);

/*
 * Aggregation with the activation sigma of eq. (4) applied on the way out, for the two places where
 * an epoch applies it right after an aggregation (no separate pass over the matrix):
 *   - a layer evaluated as sigma(A_hat (H W)) (transform first, aggregate at the narrower output
 *     width): direction NTP_FWD, act NTP_ACT_RELU, M NULL:   Y = max(A_hat X, 0);
 *   - the gradient that flows back into a ReLU layer through the aggregation above it:
 *     direction NTP_BWD, act NTP_ACT_RELU, M = that layer's output H [n x f_slice], row stride ldm:
 *         Y = (A_hat^T X) * 1[M > 0]
 *     i.e. Y is dZ of the layer below, and its ntp_nn_bwd runs with NTP_ACT_NONE.
 * In general: an output element is kept where its mask element (the same position of M, or the
 * output itself when M is NULL) is > 0 and stored as zero elsewhere (a NaN mask element stores 0).
 * act NTP_ACT_NONE is ntp_chunked_aggregate.  M: device, same dtype as Y, must not overlap Y.
 * Chunk schedule, streams and every other rule as for ntp_chunked_aggregate (copy_stream may be
 * NULL when every chunk is resident).  Not available for the backward of a graph built with
 * NTP_SCATTER_BWD (NTP_EUNSUPPORTED).
 */
int ntp_aggregate_act(ntp_graph_t* g, int direction, const void* X, void* Y,
                      int64_t f_slice, int64_t ldx, int64_t ldy, int dtype,
                      int act, const void* M, int64_t ldm, void* compute_stream, void* copy_stream);

/*
 * Edge attention weights of GAT-style aggregation (AGG of GAT, Section 2.1; Section 4.1 computes
 * the coefficients of all edges before the aggregation starts and then aggregates with them as
 * edge weights).  For every stored entry u -> v of g (self loops included; g's own weights are
 * not used):
 *     e(u -> v)     = LeakyReLU(p[u] + q[v])              (negative_slope for e < 0)
 *     alpha(u -> v) = exp(e(u -> v)) / sum over the in-edges u' -> v of exp(e(u' -> v))
 * p[u] = a_src . (W h_u) and q[v] = a_dst . (W h_v) are the two halves of a^T [W h_u || W h_v]:
 * contiguous device fp32 arrays of n_vertices (the outputs of ntp_attention_scores_fwd).
 * alpha_in  [nnz] device fp32: the weights in the entry order of the by-destination form
 *           (ntp_graph_export(NTP_CSR)): what ntp_aggregate_weighted(NTP_FWD) takes.
 * alpha_out [nnz] device fp32, nullable: the same numbers (bit for bit) in the entry order of
 *           the by-source form: what ntp_aggregate_weighted(NTP_BWD) takes.
 * Needs every chunk of the topology device-resident (NTP_EBUDGET otherwise); alpha_out is not
 * available for graphs built with NTP_SCATTER_BWD (NTP_EUNSUPPORTED).  Deterministic.  The
 * handle keeps 16 bytes per vertex of scratch from the first call on; calls on one handle must
 * not overlap.
 */
int ntp_edge_softmax(ntp_graph_t* g, const float* p, const float* q, float negative_slope,
                     float* alpha_in, float* alpha_out, void* stream);

/*
 * Gradient of the scores p, q through the attention weights of ntp_edge_softmax, for the weighted
 * aggregation Y[v,:] = sum over in-edges u -> v of alpha(u -> v) Z[u,:] (the backward counterpart
 * of the edge-associated computation of Section 4.1, chained through the softmax and LeakyReLU of
 * the GAT aggregation of Section 2.1).  With dY = dLoss/dY:
 *     dalpha(u -> v) = dY[v,:] . Z[u,:]
 *     t[v]           = sum over in-edges of alpha dalpha
 *     de(u -> v)     = alpha (dalpha - t[v])
 *     ds(u -> v)     = de * (1 if p[u] + q[v] > 0 else negative_slope)
 *     dq[v] = sum over the in-edges of v of ds,   dp[u] = sum over the out-edges of u of ds.
 * (The gradient with respect to Z itself is ntp_aggregate_weighted(NTP_BWD, alpha_out, dY).)
 * p, q [n] device fp32: the scores the weights were computed from; alpha_in, alpha_out [nnz]: both
 * outputs of ntp_edge_softmax; Z, dY [n x m] device fp32, row strides ldz, lddy >= m,
 * 1 <= m <= 1024 when both are 16-byte aligned with m and the strides multiples of 4, m <= 256
 * otherwise (NTP_EUNSUPPORTED); dp, dq [n] device fp32 outputs: every element written when
 * accumulate is 0, every element added to when it is not (the same weights used by several
 * aggregation rounds, Section 4.1: one call per round, the first with accumulate = 0).
 * Needs every chunk device-resident (NTP_EBUDGET) and a by-source form (NTP_EUNSUPPORTED for
 * NTP_SCATTER_BWD graphs).  On a graph built with NTP_EDGE_PERM the by-source pass is a one-column
 * aggregation of per-edge values through the permutation instead of a second round of dot products
 * (same result to rounding).  Deterministic.  The handle keeps 4 bytes per edge + 12 per vertex of
 * scratch from the first call on; calls on one handle must not overlap.
 */
int ntp_edge_softmax_bwd(ntp_graph_t* g, const float* p, const float* q, float negative_slope,
                         const float* alpha_in, const float* alpha_out, const float* Z, const float* dY,
                         int64_t m, int64_t ldz, int64_t lddy, float* dp, float* dq, int accumulate, void* stream);

/*
 * The vertex-associated half of the attention of Section 2.1: a^T [W h_u || W h_v] is
 * p[u] + q[v] with p[v] = Z[v,:] . a_src and q[v] = Z[v,:] . a_dst, Z = the transformed embeddings
 * (the rows W h_v).  Both products from one read of Z.
 * Z [n x m] device fp32, row stride ldz >= m, 1 <= m <= 1024; a_src, a_dst [m] device fp32;
 * p, q [n] device fp32 outputs (what ntp_edge_softmax takes).  Deterministic.
 */
int ntp_attention_scores_fwd(const float* Z, const float* a_src, const float* a_dst, float* p, float* q,
                             int64_t n, int64_t m, int64_t ldz, void* stream);

/*
 * Chain rule through ntp_attention_scores_fwd, given dp, dq [n] (from ntp_edge_softmax_bwd):
 *     dZ[v,:] += dp[v] a_src + dq[v] a_dst        (added to what dZ holds: the gradient that
 *                                                  reached Z along the aggregation)
 *     da_src = Z^T dp,   da_dst = Z^T dq           ([m] device fp32 outputs, overwritten)
 * dZ [n x m] device fp32 in/out, row stride lddz >= m; must not alias Z.  scratch: device memory of
 * at least ntp_attention_scores_bwd_scratch_bytes(n, m) bytes (at most 4 MiB), contents
 * irrelevant before and after.  Column sums are taken in a fixed order: deterministic.
 */
int ntp_attention_scores_bwd(const float* Z, const float* a_src, const float* a_dst, const float* dp, const float* dq,
                             float* dZ, float* da_src, float* da_dst, int64_t n, int64_t m, int64_t ldz, int64_t lddz,
                             void* scratch, int64_t scratch_bytes, void* stream);
int64_t ntp_attention_scores_bwd_scratch_bytes(int64_t n, int64_t m);

/*
 * ntp_aggregate_fwd / ntp_aggregate_bwd with caller-supplied edge weights in place of the
 * stored ones (gamma of Section 4.1: attention weights, or any per-edge weight):
 *   NTP_FWD: Y[v,:] = sum over entries k of row v of the by-destination form  weights[k] X[colidx[k],:]
 *   NTP_BWD: the product with the by-source form; weights in that form's entry order.  On a
 *            graph built with NTP_SCATTER_BWD the backward scatters along the by-destination
 *            rows and takes the weights in by-destination order.
 * weights: device fp32 [nnz].  Everything else as for ntp_aggregate_fwd.
 */
int ntp_aggregate_weighted(ntp_graph_t* g, int direction, const float* weights, const void* X, void* Y,
                           int64_t f_slice, int64_t ldx, int64_t ldy, int dtype, void* stream);

/*
 * Dense transform, UPDATE of eq. (4):  H = act(A W),  A [n x k] (ld k), W [k x m] (ld m),
 * H [n x m] (ld m), all device, row-major, dtype NTP_F32 or NTP_BF16 (bf16 operands on the
 * bf16 matrix instructions, fp32 accumulate, bf16 output).  act = NTP_ACT_NONE or NTP_ACT_RELU.
 * Arithmetic of NTP_F32: products with a contraction of at least 64 and an output of at least
 * 64 columns run on the bf16 matrix instructions with every fp32 operand cut exactly into three
 * bf16 pieces (hi + mid + lo) and the six piece products of weight >= 2^-16 accumulated in
 * fp32: each product a*b is formed to within 2^-23 |a b|, the accuracy of an fp32 multiply-add
 * chain, at several times the fp32 matrix rate.  One difference from fp32 arithmetic: an input
 * that is +-inf gives NaN (inf - inf in the cut) where an fp32 product would give inf.
 * Narrower or shorter products run on the fp32 matrix instructions.  The same holds for
 * ntp_nn_bwd.  (NTP_NN_CORE=fp32 in the environment selects the fp32 instructions throughout.)
 */
int ntp_nn_fwd(const void* A, const void* W, void* H, int64_t n, int64_t k, int64_t m,
               int act, int dtype, void* stream);

/*
 * Gradients of the dense transform (UPDATE in the reverse loop of Alg. 1):
 *   dZ = dH * 1[H > 0] for NTP_ACT_RELU (else dH);  dW = A^T dZ [k x m] (overwritten, always
 *   fp32; skipped when dW is NULL);  dA = dZ W^T [n x k] (skipped when dA is NULL).  At least
 *   one of the two must be given: a caller may ask for them in two calls on two streams, e.g.
 *   dA on the stream that continues with the backward aggregation and dW beside it.
 * workspace: device scratch of at least ntp_nn_bwd_workspace_bytes(n,k,m) bytes, caller
 * owned (holds the partial sums of the reduction over n; not needed when dW is NULL).
 */
int ntp_nn_bwd(const void* A, const void* W, const void* H, const void* dH,
               void* dA, float* dW, int64_t n, int64_t k, int64_t m,
               int act, int dtype, void* workspace, int64_t workspace_bytes, void* stream);

int64_t ntp_nn_bwd_workspace_bytes(int64_t n, int64_t k, int64_t m);

/*
 * Loss of the vertex classification task that closes the forward loop of Alg. 1 and starts the
 * reverse loop:  loss[0] = mean over the n vertices of -log softmax(Z[v, 0:c])[labels[v]]  and
 * dZ[v, :] = (softmax(Z[v, :]) - onehot(labels[v])) / n.  Z, dZ: device fp32, row strides ldz,
 * lddz >= c, not overlapping; labels: device int64, a label
 * outside [0, c) contributes no loss and no -1; loss: one device float.  scratch: device memory
 * of ntp_softmax_xent_scratch_bytes(n) bytes, caller owned.  Deterministic (fixed-order sums).
 */
int ntp_softmax_xent(const float* Z, const int64_t* labels, float* dZ, float* loss,
                     void* scratch, int64_t scratch_bytes, int64_t n, int64_t c,
                     int64_t ldz, int64_t lddz, void* stream);
int64_t ntp_softmax_xent_scratch_bytes(int64_t n);

/*
 * The activation sigma of eq. (4) on its own, for a layer evaluated as sigma(A_hat (H W))
 * (transform first, aggregate at the narrower output width, then activate), where it cannot
 * be fused into the transform.  ntp_relu_fwd: H = max(H, 0) in place.  ntp_relu_bwd:
 * dZ = dH where H > 0, else 0 (dZ may be dH itself).  H, dH, dZ: device, [n x f], common row
 * stride ld (elements), dtype NTP_F32 or NTP_BF16.  Asynchronous on `stream`.
 */
int ntp_relu_fwd(void* H, int64_t n, int64_t f, int64_t ld, int dtype, void* stream);
int ntp_relu_bwd(const void* dH, const void* H, void* dZ, int64_t n, int64_t f, int64_t ld,
                 int dtype, void* stream);

/* Release a graph: waits for the device, frees device, pinned and host memory. NULL ok. */
void ntp_graph_free(ntp_graph_t* g);

/* Text of the last error raised on this thread ("" if none). Valid until the next call. */
const char* ntp_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* NTP_H */
