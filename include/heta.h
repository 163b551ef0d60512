/*
 * heta.h - C ABI of the MI355X (gfx950) library for the data-parallel hot path of the
 * Relation-Aggregation-First (RAF) heterogeneous-GNN layer of arXiv 2408.09697.
 *
 * What the path computes (Eq. 1 of the paper with AGG_r = GCN-style neighbour sum/mean
 * times a per-relation weight matrix, AGG_all = sum; Section 2.1):
 *
 *     M_r[v] = (sum | mean) over edges e of relation r into v of H0_s[u_e]      aggregate
 *     Z_r    = M_r . W_r                                                        project
 *     H_t    = sum over relations r into type t of Z_r                          cross-relation
 *
 * and the backward pass of Algorithm 1's local backpropagation:
 *
 *     dZ_r = G_t ;  dW_r = M_r^T dZ_r ;  dM_r = dZ_r W_r^T ;
 *     dH0_s[u] += sum over edges e of r out of u of c_e dM_r[v_e],  c_e = 1 | 1/deg_r(v_e)
 *
 * Conventions for every call
 *   - "device" pointers are HIP device memory of the current device; "host" pointers are
 *     ordinary process memory.  The library never takes ownership of a caller's buffer and
 *     never frees one.  It owns only heta_graph handles and what hangs off them.
 *   - Matrices are row-major with a leading dimension `ld` counted in ELEMENTS.
 *   - Every compute call is asynchronous on the given HIP stream (`hip_stream` is a
 *     hipStream_t passed as void*, NULL = the default stream) and performs no hidden
 *     synchronisation, except where a call says it may grow the handle's workspace.
 *   - Every call returns a heta_status.  Arguments are validated on the host before any
 *     kernel is launched; on failure nothing is launched, output buffers are untouched and
 *     heta_last_error() describes the reason.  No exception or abort crosses this boundary.
 *   - Results are deterministic: no atomics are used, the same inputs give the same bits.
 *   - Node ids within a type and table row numbers must be below 2^31; edge offsets are 64-bit.
 */
#ifndef HETA_H
#define HETA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct heta_graph heta_graph; /* opaque, created and destroyed by the library */

typedef enum {
    HETA_OK = 0,
    HETA_ERR_INVALID_ARG = 1, /* null pointer, negative size, unknown enum value, index out of range */
    HETA_ERR_BAD_CSR = 2,     /* rowptr not monotone / not starting at 0 / not ending at E, column out of range */
    HETA_ERR_SHAPE = 3,       /* ld < d, widths that do not fit, beta other than 0 or 1 where required */
    HETA_ERR_UNSUPPORTED = 4, /* dtype combination or size the library has no kernel for */
    HETA_ERR_OOM = 5,         /* host or device allocation failed */
    HETA_ERR_DEVICE = 6       /* a HIP call failed; heta_last_error() carries the HIP message */
} heta_status;

typedef enum { HETA_F32 = 0, HETA_BF16 = 1 } heta_dtype;
typedef enum { HETA_SUM = 0, HETA_MEAN = 1 } heta_reduce;
typedef enum { HETA_ACT_NONE = 0, HETA_ACT_RELU = 1 } heta_act;

/* flags of heta_graph_create */
#define HETA_PTRS_ON_DEVICE 1u /* the index arrays of every heta_relation are device pointers */

/* A node type (Section 2.1: each node type may carry feature vectors of its own width, or
 * none, in which case it gets learnable vectors).  feat_dim and learnable are descriptive;
 * tables are passed to the compute calls. */
typedef struct {
    int64_t num_nodes;
    int32_t feat_dim;
    int32_t learnable;
} heta_ntype;

/* A relation = one mono-relation subgraph (Section 2.1), a bipartite adjacency from
 * src_type to dst_type given as a CSR over DESTINATION rows, optionally with its CSC.
 *
 * csc_colptr / csc_row (both or neither; NULL = the library derives them): the transposed adjacency,
 * column u listing the destinations of u's out-edges in ascending original edge position, which for a
 * CSR means in non-decreasing order.  That order makes the CSC unique; the library checks a supplied
 * CSC against the one it derives from the CSR, element by element, and rejects any difference with
 * HETA_ERR_BAD_CSR (a backward pass over a CSC that disagreed with the CSR would silently compute the
 * gradient of another graph).  The check costs what deriving costs, so supplying a CSC saves nothing.
 *
 * reverse_of (-1 = none; else the index j < i of an earlier relation of the same array): declares this
 * relation to be the exact transpose of relation j - source and destination types swapped, the same
 * edges, its CSR equal to relation j's CSC element by element (checked: HETA_ERR_BAD_CSR otherwise).
 * The graphs of the paper's evaluation list every relation with its reverse.  A declared reverse shares
 * relation j's index arrays and row schedules (its CSR is j's CSC, its CSC is j's CSR) instead of
 * holding copies: half the index memory of the pair.  Results are those of an undeclared reverse.
 * Zero-initialise the struct and set reverse_of = -1 when the fields are not used. */
typedef struct {
    int32_t src_type, dst_type;
    int64_t num_edges;
    const int64_t *csr_rowptr; /* [n_dst + 1], rowptr[0] = 0, non-decreasing, rowptr[n_dst] = num_edges */
    const int32_t *csr_col;    /* [num_edges] source node ids in [0, n_src); any order, duplicates allowed */
    const int64_t *csc_colptr; /* [n_src + 1] or NULL */
    const int32_t *csc_row;    /* [num_edges] destination node ids, or NULL */
    int32_t reverse_of;        /* -1, or the index of the relation this one is the transpose of */
} heta_relation;

/* ---- graph ingest (HetG and its decomposition into mono-relation subgraphs, Section 2.1) ------
 * Validates every relation, copies its CSR to the device, computes in-degrees, builds the
 * transposed adjacency (CSC: for each source u the destinations of its out-edges in ascending
 * original edge position) and the degree-sorted row schedules both directions use (device
 * kernels: a stable radix sort of (source, destination) pairs, scans, binary searches).
 * Synchronous.  The caller's arrays may be freed on return.  `*out` is written only on success.
 * Where a CSR is checked: host arrays of a relation that is uploaded and built on its own are walked on
 * the host first; device arrays (HETA_PTRS_ON_DEVICE), and the small relations of a graph that are built
 * together on the device (a sampled block's), are checked by the build's own kernels - the same findings,
 * HETA_ERR_BAD_CSR, and no handle, but only after those kernels ran. */
heta_status heta_graph_create(const heta_ntype *ntypes, int32_t n_ntypes, const heta_relation *rels,
                              int32_t n_rels, uint32_t flags, heta_graph **out);
/* Several graphs at once - the blocks of one sampled mini-batch (Algorithm 1 samples one block per layer
 * and iteration): the same handles as n_graphs calls of heta_graph_create, array for array, but the small
 * relations of all of them are built by one set of device kernels (one block-diagonal problem), so a
 * mini-batch pays the launch chain of its block handles once instead of once per layer.  ntypes / n_ntypes /
 * rels / n_rels: HOST arrays of n_graphs entries, each as for heta_graph_create; flags apply to all graphs;
 * out: HOST array of n_graphs handles, all NULL on failure.  The handles are independent afterwards (each is
 * destroyed on its own; memory the blocks share goes with the last).  Relations beyond what one build takes
 * (32 small relations in all), or too few edges for the device to pay, are built graph by graph. */
heta_status heta_graph_create_batch(int32_t n_graphs, const heta_ntype *const *ntypes, const int32_t *n_ntypes,
                                    const heta_relation *const *rels, const int32_t *n_rels, uint32_t flags,
                                    heta_graph **out);
heta_status heta_graph_destroy(heta_graph *g); /* NULL is accepted; synchronises the device */
/* Device bytes the handle holds for index data (adjacency in both directions, schedules, 1/deg);
 * arrays shared through reverse_of count once. */
heta_status heta_graph_index_bytes(const heta_graph *g, int64_t *bytes);

/* Read-back of the derived index data into HOST buffers (for bit-exact checks). Synchronous.  The CSC
 * comes back in its unique order (rows of a column non-decreasing) also for a relation that shares
 * another one's arrays. */
heta_status heta_graph_get_csc(const heta_graph *g, int32_t rel, int64_t *colptr /* [n_src+1] */,
                               int32_t *row /* [num_edges] */);
heta_status heta_graph_get_degrees(const heta_graph *g, int32_t rel, int64_t *in_deg /* [n_dst] */);

/* ---- heterogeneous gather: h^0 of a node type from its feature or learnable table -------------
 * (Section 2.1: h^0_v is the feature vector of v, or its learnable vector.)
 * out[i, 0:d] = table[gid[i], 0:d] for i < n; bit-exact copy.  All pointers device.
 * gid entries must lie in [0, n_table_rows): heta_check_ids can verify that. */
heta_status heta_feature_gather(const void *table, heta_dtype dt, int64_t ld_table, int32_t d,
                                int64_t n_table_rows, const int64_t *gid, int64_t n, void *out,
                                int64_t ld_out, void *hip_stream);
/* Counts entries of a device int64 id array outside [0, limit); synchronises the stream.
 * Returns HETA_ERR_INVALID_ARG when any is out of range. */
heta_status heta_check_ids(const int64_t *ids, int64_t n, int64_t limit, void *hip_stream);

/* ---- relation-specific aggregation, forward (Eq. 1, first line; Algorithm 1, the workers'
 * "aggregate neighbour features/embeddings" step) ------------------------------------------------
 * out[v, 0:d] = sum over e in CSR row v of src_table[row(col[e]), 0:d], row(u) = src_gid ? src_gid[u] : u;
 * HETA_MEAN divides by the row's degree; a zero-degree row gives exactly 0.
 * src_table: device [n_table_rows, ld_src] of in_dt; needs n_table_rows >= n_src when src_gid is NULL.
 * src_gid:   device [n_src] or NULL (local -> table row map of a sampled block; entries unchecked).
 * out:       device [n_dst, ld_out] of out_dt (fp32 accumulation either way); beta = 1 adds the result
 *            to what out holds (a relation's aggregate accumulated straight into H_t), beta = 0 overwrites.
 * Rows with ld * sizeof(elem) a multiple of 16 and 16-byte aligned bases use 128-bit loads; anything
 * else runs an element-wise kernel, never an error.  May grow the handle's workspace when the
 * relation has rows of 512+ edges (first call for a wider d: hipMalloc, which synchronises). */
heta_status heta_rel_aggregate_fwd(heta_graph *g, int32_t rel, heta_reduce op, const void *src_table,
                                   heta_dtype in_dt, int64_t ld_src, int32_t d, int64_t n_table_rows,
                                   const int64_t *src_gid, void *out, heta_dtype out_dt, int64_t ld_out,
                                   float beta, void *hip_stream);

/* The same operation for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): identical arguments, kernels and results, but
 * the partial sums of rows with 512+ edges go to a fixed array of HETA_NOALLOC_SCRATCH_BYTES that the
 * library's code object holds on every device (until the process ends) instead of the handle's
 * grow-on-demand workspace.  The call performs no hipMalloc / hipFree and creates no events (its
 * launches are not seen by heta_profile_*).  The array's address is looked up once per device, by
 * heta_graph_create or else by the first call.  A relation whose partials do not fit
 * (ceil(E_hub / 256 + hub rows) * round8(d) * 4 bytes, E_hub = edges in rows of 512+ edges) returns
 * HETA_ERR_UNSUPPORTED with nothing launched.  All calls on one device share the array: calls that
 * overlap in time on one GPU (different streams or threads) race; keep them stream-ordered. */
#define HETA_NOALLOC_SCRATCH_BYTES (32u << 20)
heta_status heta_rel_aggregate_fwd_noalloc(heta_graph *g, int32_t rel, heta_reduce op, const void *src_table,
                                           heta_dtype in_dt, int64_t ld_src, int32_t d, int64_t n_table_rows,
                                           const int64_t *src_gid, void *out, heta_dtype out_dt, int64_t ld_out,
                                           float beta, void *hip_stream);

/* ---- relation-specific aggregation, backward (Algorithm 1, local backpropagation with the
 * gradients of the partial aggregations) ---------------------------------------------------------
 * grad_src[u, 0:d] = beta * grad_src[u, 0:d] + sum over e in CSC column u of c_e * grad_out[row[e], 0:d]
 * c_e = 1 (HETA_SUM) or 1/deg_r(row[e]) (HETA_MEAN).  A gather over the CSC: no atomics.
 * grad_out: device [n_dst, ld_go] of go_dt (fp32, or bf16 when the caller keeps dM_r in the
 * storage type; accumulation is fp32 either way); grad_src: device fp32 [n_src, ld_gs]; beta is
 * 0 or 1 (1 accumulates the relations that share a source type, in the caller's call order). */
heta_status heta_rel_aggregate_bwd(heta_graph *g, int32_t rel, heta_reduce op, const void *grad_out,
                                   heta_dtype go_dt, int64_t ld_go, int32_t d, float *grad_src, int64_t ld_gs,
                                   float beta, void *hip_stream);

/* ---- several relations per launch (Algorithm 1: a worker aggregates every relation of its partition;
 * the relation-specific aggregations of one layer are independent of each other) ------------------
 * One item is one heta_rel_aggregate_fwd / heta_rel_aggregate_bwd call; a call with n items computes
 * exactly what the n single calls compute (same kernels, same summation order, bitwise the same
 * results), but items that take the same kernel (same dtype, same d, same alignment class) share
 * launches of up to four relations.  For the small relations of a sampled mini-batch block, where a
 * launch costs more than its work, this is the difference between n launch latencies and n / 4.
 * The items of one call run concurrently: no two may write overlapping outputs (checked; a type that
 * is the source of two relations takes its two backward items in two calls, beta = 0 then beta = 1).
 *   forward : in = src_table [n_table_rows, ld_in] of in_dt, src_gid as in heta_rel_aggregate_fwd,
 *             out [n_dst, ld_out] of out_dt
 *   backward: in = grad_out [n_dst, ld_in] of in_dt; out = grad_src, fp32 [n_src, ld_out];
 *             n_table_rows and src_gid are ignored
 * items: host array, read before the call returns.  n = 0 is a no-op.  Errors as the single calls,
 * detected before anything is launched. */
typedef struct heta_agg_item {
    int32_t rel;
    int32_t d;
    const void *in;          /* device */
    int64_t ld_in;
    int64_t n_table_rows;
    const int64_t *src_gid;  /* device or NULL */
    void *out;               /* device */
    int64_t ld_out;
    float beta;              /* 0 or 1 */
} heta_agg_item;
heta_status heta_rel_aggregate_fwd_multi(heta_graph *g, int32_t n, const heta_agg_item *items, heta_reduce op,
                                         heta_dtype in_dt, heta_dtype out_dt, void *hip_stream);
heta_status heta_rel_aggregate_bwd_multi(heta_graph *g, int32_t n, const heta_agg_item *items, heta_reduce op,
                                         heta_dtype in_dt, void *hip_stream);

/* ---- per-relation projection (the per-relation weight matrices of R-GCN, Section 2.1) ---------
 * out[i, 0:d_out] = beta * out[i, 0:d_out] + s_i * sum_k in[i, k] * B[k, j],  i < n_rows,
 *   B = W          (W is [d_in, d_out], ld_w >= d_out)   when transW == 0     (forward,  Z = M W)
 *   B = W^T        (W is [d_out, d_in], ld_w >= d_in)    when transW != 0     (backward, dM = dZ W^T)
 *   s_i = row_scale ? row_scale[i] : 1.
 * in: device [n_rows, ld_in] of in_dt; W device of w_dt; out device [n_rows, ld_out] of out_dt
 * (fp32, or bf16 for an intermediate kept in the storage type: then beta must be 0 and row_scale NULL).
 * Both fp32 -> fp32 MFMA; otherwise operands are rounded to bf16 and multiplied on the bf16 MFMA
 * path; accumulation is fp32 in both.  beta = 1 fuses the cross-relation sum into the projection.
 * heta_rel_project takes n_rows = n_dst of the relation; heta_project any row count.  The handle is not
 * const: with bf16 weights the call may grow its packing buffer (see heta_cross_rel_project). */
heta_status heta_project(int64_t n_rows, const void *in, heta_dtype in_dt, int64_t ld_in, int32_t d_in,
                         const void *W, heta_dtype w_dt, int64_t ld_w, int32_t d_out, int32_t transW,
                         const float *row_scale, void *out, heta_dtype out_dt, int64_t ld_out, float beta,
                         void *hip_stream);
heta_status heta_rel_project(heta_graph *g, int32_t rel, const void *in, heta_dtype in_dt,
                             int64_t ld_in, int32_t d_in, const void *W, heta_dtype w_dt, int64_t ld_w,
                             int32_t d_out, int32_t transW, const float *row_scale, void *out,
                             heta_dtype out_dt, int64_t ld_out, float beta, void *hip_stream);

/* Weight gradient dW[0:d_in, 0:d_out] = beta * dW + in^T . gout, the sum running over the n_dst
 * rows of the relation in a fixed order (split over workgroups, then combined in order).
 * in: device [n_dst, ld_in] of in_dt (the saved M_r); gout: device fp32 [n_dst, ld_go];
 * dW: device fp32 [d_in, ld_dw].  Uses the handle's workspace (may grow it, see above). */
heta_status heta_rel_project_wgrad(heta_graph *g, int32_t rel, const void *in, heta_dtype in_dt,
                                   int64_t ld_in, int32_t d_in, const float *gout, int64_t ld_go,
                                   int32_t d_out, float *dW, int64_t ld_dw, float beta, void *hip_stream);

/* ---- several projections in one launch (the same per-relation weight matrices; used when relations
 * are projected before they are aggregated, which Eq. 1's linearity allows) --------------------------
 * heta_project_batch: outs[p] = ins[p] . (Ws[p] or Ws[p]^T) for p < n (1..8), independent products
 *   scheduled so that operands several of them share (e.g. one source table under the weights of all
 *   its outgoing relations) are fetched from HBM once.  outs[p] device [n_rows, ld_out[p]] of out_dt.
 * heta_project_sum:   out = beta * out + sum_p ins[p] . (Ws[p] or Ws[p]^T), one contraction over the
 *   concatenated k ranges (e.g. a source type's input gradient summed over its outgoing relations).
 * heta_project_wgrad_batch: dW[p] = beta * dW[p] + ins[p]^T . gouts[p] over n_rows rows, every p with
 *   its own gradient operand; uses the handle's workspace; gout_two_terms as in
 *   heta_cross_rel_project_wgrad.
 * Pointer and size arrays are HOST arrays of n entries; shapes and dtypes as in heta_project.
 * g (heta_project_batch, heta_project_sum): optional (NULL allowed) handle whose packing buffer the call may use
 *   to rewrite the weights into the form its kernel reads fastest (fp32 weights as three bf16 terms), on the
 *   same terms as heta_cross_rel_project; the result does not depend on it beyond rounding order. */
heta_status heta_project_batch(heta_graph *g, int64_t n_rows, int32_t n, const void *const *ins, heta_dtype in_dt, const int64_t *ld_in,
                               const int32_t *d_in, const void *const *Ws, heta_dtype w_dt, const int64_t *ld_w,
                               int32_t d_out, int32_t transW, void *const *outs, heta_dtype out_dt,
                               const int64_t *ld_out, void *hip_stream);
heta_status heta_project_sum(heta_graph *g, int64_t n_rows, int32_t n, const void *const *ins, heta_dtype in_dt, const int64_t *ld_in,
                             const int32_t *d_in, const void *const *Ws, heta_dtype w_dt, const int64_t *ld_w,
                             int32_t d_out, int32_t transW, float *out, int64_t ld_out, float beta, void *hip_stream);
heta_status heta_project_wgrad_batch(heta_graph *g, int64_t n_rows, int32_t n, const void *const *ins, heta_dtype in_dt,
                                     const int64_t *ld_in, const int32_t *d_in, const float *const *gouts,
                                     const int64_t *ld_go, int32_t d_out, float *const *dW, const int64_t *ld_dw,
                                     float beta, int32_t gout_two_terms, void *hip_stream);

/* ---- projection of all relations into one destination type, fused with the cross-relation sum --
 * (Eq. 1, both lines in one pass; Algorithm 1, relation-specific aggregation followed by AGG_all.)
 * out[i, 0:d_out] = act(beta * out[i, 0:d_out] + sum_{p<n} ins[p][i, 0:d_in[p]] . Ws[p]),  i < n_rows(dst_type):
 * one contraction over the concatenated k ranges, so no per-relation partial ever goes to HBM.
 * ins, Ws, ld_in, d_in, ld_w: HOST arrays of n (1..8) entries; ins[p] device [n_rows, ld_in[p]] of
 * in_dt; Ws[p] device [d_in[p], ld_w[p] >= d_out] of w_dt; out device fp32 [n_rows, ld_out].
 * On a subset of a type's relations with beta = 0 it yields the partial aggregation of that subset.
 * With bf16 inputs and weights the call first rewrites the weights k-contiguous into a buffer of the
 * handle (grown on demand: the first call for a larger shape synchronises); with fp32 inputs and weights
 * and enough rows for full-size tiles it rewrites the weights there as the three bf16 terms the product is
 * fed with (so does heta_cross_rel_project_bwd).  Calls on one handle that do so must be stream-ordered,
 * like the calls that use its workspace. */
heta_status heta_cross_rel_project(heta_graph *g, int32_t dst_type, int32_t n, const void *const *ins,
                                   heta_dtype in_dt, const int64_t *ld_in, const int32_t *d_in,
                                   const void *const *Ws, heta_dtype w_dt, const int64_t *ld_w, int32_t d_out,
                                   heta_act act, float *out, int64_t ld_out, float beta, void *hip_stream);
/* Its backward, one launch each for all n relations into dst_type (Algorithm 1, local
 * backpropagation): dM[p] = gout . Ws[p]^T and dW[p] = beta * dW[p] + ins[p]^T . gout.
 * gout device fp32 [n_rows, ld_go]; dM[p] device [n_rows, ld_dm[p] >= d_in[p]] of dm_dt (fp32, or
 * bf16: the fp32 accumulator is rounded once on the way out, for callers that store the [n x d]
 * intermediates of a layer in the storage type); dW[p] device fp32 [d_in[p], ld_dw[p] >= d_out];
 * the pointer arrays are HOST arrays.
 * The wgrad call uses the handle's workspace (may grow it, see heta_rel_aggregate_fwd).  With bf16
 * inputs gout is rounded to bf16 for the MFMA; gout_two_terms != 0 feeds it as two bf16 terms (the
 * rounded value and what the rounding left: 16 significant bits) - for a gout that was itself
 * summed over many edges, whose magnitude makes a single rounding visible in dW. */
heta_status heta_cross_rel_project_bwd(const heta_graph *g, int32_t dst_type, int32_t n, const float *gout,
                                       int64_t ld_go, int32_t d_out, const void *const *Ws, heta_dtype w_dt,
                                       const int64_t *ld_w, const int32_t *d_in, void *const *dM,
                                       heta_dtype dm_dt, const int64_t *ld_dm, void *hip_stream);
heta_status heta_cross_rel_project_wgrad(heta_graph *g, int32_t dst_type, int32_t n, const void *const *ins,
                                         heta_dtype in_dt, const int64_t *ld_in, const int32_t *d_in,
                                         const float *gout, int64_t ld_go, int32_t d_out, float *const *dW,
                                         const int64_t *ld_dw, float beta, int32_t gout_two_terms, void *hip_stream);

/* ---- fused forward for inference: aggregation, projection and cross-relation sum in one kernel (Eq. 1,
 * both lines; Algorithm 1, the aggregation and AGG_all steps), the aggregated features never reach HBM:
 *   out[v, 0:d_out] = act( sum_{p < n} ( (sum|mean)_{e in rels[p], v_e = v} table_p[row(u_e)] ) W_p ).
 * rels: HOST array of n (1..16) relations, all ending in dst_type; tables, ld_table, d_table (width of
 * table_p = rows of W_p), n_table_rows, src_gid (nullable array, nullable entries), W, ld_w: HOST arrays of
 * n entries as in heta_rel_aggregate_fwd / heta_rel_project; tables and W share the element type dt.
 * out: device fp32 [n_rows(dst_type), ld_out], overwritten.
 * HETA_ERR_UNSUPPORTED (nothing launched) unless d_out <= 256 and every source row is a 16-byte aligned
 * multiple of 16 bytes: use the unfused calls then.  Training needs the aggregated features for the
 * weight gradient and uses the unfused calls as well. */
heta_status heta_cross_rel_aggregate_project(heta_graph *g, int32_t dst_type, int32_t n, const int32_t *rels,
                                             heta_reduce op, const void *const *tables, heta_dtype dt,
                                             const int64_t *ld_table, const int32_t *d_table, const int64_t *n_table_rows,
                                             const int64_t *const *src_gid, const void *const *W, const int64_t *ld_w,
                                             int32_t d_out, heta_act act, float *out, int64_t ld_out, void *hip_stream);

/* ---- cross-relation aggregation (Eq. 1, second line; Algorithm 1, AGG_all on the designated
 * worker; on a subset of relations it yields the partial aggregation a worker would send) --------
 * out[i, 0:d_out] = act(sum_{p < n_partials} partials[p][i, 0:d_out]), summed in array order.
 * partials: HOST array of n_partials (1..16) device pointers, each fp32 [n_rows(dst_type), ld];
 * out: device fp32 [n_rows, ld_out]; out may alias partials[0]. */
heta_status heta_cross_rel_reduce(const heta_graph *g, int32_t dst_type, const float *const *partials,
                                  int32_t n_partials, int64_t ld, int32_t d_out, heta_act act,
                                  float *out, int64_t ld_out, void *hip_stream);
/* Backward of the activation: grad_in = grad_out * [h > 0] for HETA_ACT_RELU (copy otherwise).
 * All device fp32 [n_rows, ld]; grad_in may alias grad_out. */
heta_status heta_act_bwd(int64_t n_rows, int32_t d, heta_act act, const float *h, int64_t ld_h,
                         const float *grad_out, int64_t ld_go, float *grad_in, int64_t ld_gi,
                         void *hip_stream);

/* ---- graph attention as the relation-specific aggregation (Section 2.1: R-GAT applies GAT for
 * AGG_r, sums the relations' outputs and activates the sum with ReLU; the paper prints no formula for
 * the module, so it is the attention layer of the GAT paper, Velickovic et al. 2018, Eqs. 1-4 with
 * multi-head concatenation, on a bipartite relation) ------------------------------------------------
 * With K = heads, F = d / K, z = H0_s W_r (heta_project), for every edge e = (u_e -> v_e) of `rel`:
 *   s_e[k] = LeakyReLU_slope(el[u_e, k] + er[v_e, k]);  alpha_e[k] = softmax of s_e[k] over the in-edges of v_e;
 *   out[v, kF + f] = beta out[v, kF + f] + sum_{e into v} alpha_e[k] z[u_e, kF + f].
 * Multi-edges are separate softmax terms; a destination without in-edges gets 0 (untouched when beta = 1).
 *
 * heta_attn_score: score[i, k] = sum_j x[i, j] vec_k[j].  per_head = 1: j runs over head k's columns
 *   [kF, (k+1)F) and vec is [K][F] (el = <z_u[k,:], a[k,:]>); per_head = 0: j runs over all d columns and
 *   vec is [K][d] (er = <h_v, q[k,:]>, q[k,:] being the destination-side weight matrix times its half of
 *   GAT's attention vector).  x: device [n, ld_x] of dt; vec: device fp32; score: device fp32 [n, K]. */
heta_status heta_attn_score(const void *x, heta_dtype dt, int64_t ld_x, int64_t n, int32_t d, const float *vec,
                            int32_t heads, int32_t per_head, float *score, void *hip_stream);
/* Backward of heta_attn_score: dx[i, j] = beta dx[i, j] + sum_k dscore[i, k] vec_k[j] (dx: device fp32
 * [n, ld_dx] or NULL; beta 0 or 1) and dvec_k[j] = sum_i dscore[i, k] x[i, j] (device fp32, shaped like
 * vec, overwritten, or NULL), rows added in a fixed order (partial sums in g's attention workspace). */
heta_status heta_attn_score_bwd(heta_graph *g, const void *x, heta_dtype dt, int64_t ld_x, int64_t n, int32_t d,
                                const float *vec, int32_t heads, int32_t per_head, const float *dscore, float *dx,
                                int64_t ld_dx, float beta, float *dvec, void *hip_stream);
/* The same for several vector sets over ONE table in one pass (a node type is the source of some relations
 * and the destination of others; each takes a score of the type's table with vectors of its own):
 *   scores[s][i, k] = sum_j x[i, j] vecs[s][k][j]                              (per_head = 0 semantics)
 *   dx[i, j] = beta dx[i, j] + sum_s sum_k dscores[s][i, k] vecs[s][k][j];  dvecs[s][k][j] = sum_i dscores[s][i, k] x[i, j]
 * vecs / scores / dscores / dvecs: HOST arrays of n_sets device pointers (fp32; [K][d] and [n, K]); dvecs or
 * single entries of it may be NULL, dx may be NULL.  Tables of at most 128 columns (a multiple of 4, rows
 * 16-byte aligned for fp32, 8-byte for bf16) with n_sets <= 8 and n_sets * heads <= 32 are read once; other
 * shapes are served set by set by the calls above, with the same results up to summation order. */
heta_status heta_attn_score_multi(const void *x, heta_dtype dt, int64_t ld_x, int64_t n, int32_t d, int32_t n_sets,
                                  const float *const *vecs, int32_t heads, float *const *scores, void *hip_stream);
heta_status heta_attn_score_bwd_multi(heta_graph *g, const void *x, heta_dtype dt, int64_t ld_x, int64_t n, int32_t d,
                                      int32_t n_sets, const float *const *vecs, int32_t heads, const float *const *dscores,
                                      float *dx, int64_t ld_dx, float beta, float *const *dvecs, void *hip_stream);
/* The source score taken off the input table: since z_u = W^T h_u, el[u, k] = <z_u[k,:], a[k,:]> equals
 * <h_u, wa[k,:]> with wa[k, j] = sum_f W[j, kF + f] a[k, f].  heta_attn_fold writes wa (device fp32
 * [K][d_in]); el is then heta_attn_score(H0_s, wa, per_head = 0) - read from the input table, so in the
 * bf16 storage mode the logits do not see the rounding of the stored z.
 * W: device [d_in, ld_w >= d_out] of w_dt; a: device fp32 [K][F], F = d_out / K.
 * heta_attn_fold_bwd, given dwa (device fp32 [K][d_in], the dvec of heta_attn_score_bwd), writes
 *   dW[j, kF + f] = beta dW[j, kF + f] + dwa[k, j] a[k, f]   (device fp32 [d_in, ld_dw] or NULL; beta 0 or 1)
 *   da[k, f]      = sum_j dwa[k, j] W[j, kF + f]             (device fp32 [K][F] or NULL, overwritten; fixed order). */
heta_status heta_attn_fold(const void *W, heta_dtype w_dt, int64_t ld_w, int32_t d_in, int32_t d_out, const float *a,
                           int32_t heads, float *wa, void *hip_stream);
heta_status heta_attn_fold_bwd(const void *W, heta_dtype w_dt, int64_t ld_w, int32_t d_in, int32_t d_out, const float *a,
                               int32_t heads, const float *dwa, float *dW, int64_t ld_dw, float beta, float *da,
                               void *hip_stream);
/* z: device [n_src, ld_z] of z_dt; el: device fp32 [n_src, K]; er: device fp32 [n_dst, K]; out: device
 * [n_dst, ld_out] of out_dt; smax, sinv: device fp32 [n_dst, K], receive the softmax shift and the
 * reciprocal denominator that heta_rel_attn_bwd needs (both NULL for inference).  out_pos (nullable;
 * device [n_dst, ld_pos] of out_dt; needs beta = 0) receives the same sum restricted to the edges whose
 * logit el + er is positive: with it the backward needs no gather on the destination side.
 * 1 <= K <= 16, K | d.  The per-edge weights live in g's attention workspace (grown on demand; calls on
 * one handle must be stream-ordered). */
heta_status heta_rel_attn_fwd(heta_graph *g, int32_t rel, const void *z, heta_dtype z_dt, int64_t ld_z, int32_t d,
                              int32_t heads, const float *el, const float *er, float slope, void *out,
                              heta_dtype out_dt, int64_t ld_out, float beta, float *smax, float *sinv, void *out_pos,
                              int64_t ld_pos, void *hip_stream);
/* Backward of heta_rel_attn_fwd for grad_out = dL/dout (device fp32 [n_dst, ld_go]); `o` is this
 * relation's own forward output and o_pos its out_pos (device [n_dst, ld_o] of o_dt, computed with
 * beta = 0; o_pos may be NULL, at the price of one more pass over z).  Writes
 *   dz[u, kF+f] = sum_{e out of u} alpha_e[k] grad_out[v_e, kF+f]                (device fp32 [n_src, ld_dz])
 *   del[u, k], der[v, k]: the gradients of el and er through softmax and LeakyReLU (device fp32).
 * All three are overwritten.  No atomics: dz and del come from one gather over the CSC, der from row
 * products (or, without o_pos, from a gather over the CSR). */
heta_status heta_rel_attn_bwd(heta_graph *g, int32_t rel, const void *z, heta_dtype z_dt, int64_t ld_z, int32_t d,
                              int32_t heads, const float *el, const float *er, float slope, const float *smax,
                              const float *sinv, const void *o, const void *o_pos, heta_dtype o_dt, int64_t ld_o,
                              const float *grad_out, int64_t ld_go, float *dz, int64_t ld_dz, float *del, float *der,
                              void *hip_stream);

/* ---- k-hop neighbour sampling into blocks (Section 2.2 and the sampling step of Algorithm 1: a fixed
 * number of neighbours per relation is sampled, hop by hop, for the nodes of a mini-batch; fan-outs
 * {25, 20} in Section 8.1).  Rule: all in-edges of a destination if its in-degree is at most `fanout`,
 * else `fanout` distinct edge slots uniformly without replacement (Floyd's subset algorithm on a
 * SplitMix64 stream keyed by (seed, destination id): the draw does not depend on the launch or on the
 * other destinations).
 * heta_sample_neighbors: dst_ids: device [n_dst] rows of rel's destination type (checked on the device;
 *   repeated ids are sampled alike); rowptr: device [n_dst + 1], receives the block's row offsets;
 *   src_ids: device, capacity n_dst * fanout, receives the sampled GLOBAL source ids, per destination in
 *   ascending edge slot; *n_sampled (host) = rowptr[n_dst].  1 <= fanout <= 64.  Synchronous. */
heta_status heta_sample_neighbors(const heta_graph *g, int32_t rel, const int64_t *dst_ids, int64_t n_dst, int32_t fanout,
                                  uint64_t seed, int64_t *rowptr, int64_t *src_ids, int64_t *n_sampled, void *hip_stream);
/* The source set of a block and the local ids of its edges: unique_ids (device, capacity sum(lens))
 * receives the ascending distinct values of all lists, *n_unique (host) their number, and local[l]
 * (device int32 [lens[l]]) the position of lists[l][i] in unique_ids.  lists, lens, local: HOST arrays of
 * n_lists entries (device pointers / lengths); ids must lie in [0, id_limit), id_limit <= 2^31
 * (checked on the device).  Synchronous. */
heta_status heta_unique_relabel(int32_t n_lists, const int64_t *const *lists, const int64_t *lens, int64_t id_limit,
                                int64_t *unique_ids, int64_t *n_unique, int32_t *const *local, void *hip_stream);
/* The same two operations for several relations / several id sets in one call: every stage of every item
 * is queued on the stream and the call synchronises once (a mini-batch hop is one call of each).
 * heta_sample_neighbors_batch: item i samples relation rels[i] for dst_ids[i] (device [n_dst[i]]) with
 *   seeds[i] into rowptr[i] / src_ids[i] (device, sized as above); n_sampled[i] (host) receives its count.
 *   The arrays rels, dst_ids, n_dst, seeds, rowptr, src_ids, n_sampled are HOST arrays of n entries.
 * heta_unique_relabel_batch: group j owns the lists group_ptr[j] .. group_ptr[j+1]-1 of `lists` / `lens` /
 *   `local` (host arrays of device pointers / lengths) and writes unique_ids[j] (device), n_unique[j]
 *   (host) with its own id_limit[j].  Results and errors are those of the single calls. */
heta_status heta_sample_neighbors_batch(const heta_graph *g, int32_t n, const int32_t *rels, const int64_t *const *dst_ids,
                                        const int64_t *n_dst, int32_t fanout, const uint64_t *seeds, int64_t *const *rowptr,
                                        int64_t *const *src_ids, int64_t *n_sampled, void *hip_stream);
heta_status heta_unique_relabel_batch(int32_t n_groups, const int32_t *group_ptr, const int64_t *const *lists,
                                      const int64_t *lens, const int64_t *id_limit, int64_t *const *unique_ids,
                                      int64_t *n_unique, int32_t *const *local, void *hip_stream);

/* ---- sparse update of a learnable feature table (Sections 2.2 and 6: the learnable vectors of
 * featureless node types and their optimizer states, Adam's moment and variance, are updated after
 * backpropagation; only the rows a mini-batch touched) ---------------------------------------------
 * For i < n, with r = ids ? ids[i] : i and g = grad[i, 0:d] (Adam, Kingma & Ba, Algorithm 1, step t):
 *   m[r] = beta1 m[r] + (1 - beta1) g ;  v[r] = beta2 v[r] + (1 - beta2) g^2 ;
 *   table[r] -= lr * (m[r] / (1 - beta1^t)) / (sqrt(v[r] / (1 - beta2^t)) + eps).
 * table: device [n_table_rows, ld_table] of dt (a bf16 table is widened, updated in fp32 and rounded
 * back); m, v: device fp32 [n_table_rows, ld_state]; grad: device fp32 [n, ld_grad]; ids: device
 * [n] DISTINCT rows in [0, n_table_rows) or NULL for the first n rows.  An id outside that range is
 * skipped by the kernel (nothing is read or written for it; heta_check_ids reports such ids); repeated
 * rows would race.  Rows not listed are untouched, states included.
 * `step` is the global step counter t >= 1.  One pass, asynchronous on the stream. */
heta_status heta_sparse_adam(void *table, heta_dtype dt, int64_t ld_table, int32_t d, int64_t n_table_rows,
                             float *m, float *v, int64_t ld_state, const int64_t *ids, int64_t n,
                             const float *grad, int64_t ld_grad, float lr, float beta1, float beta2, float eps,
                             int64_t step, void *hip_stream);
/* The same update for several tables in one call with one set of hyper-parameters and one step counter (the weight
 * matrices of a model, ids = NULL, and its learnable tables after one backward pass): item i is what
 * heta_sparse_adam(items[i]...) would do, bit for bit; tables of different items must not overlap.  All items are
 * checked before anything is launched.  items: HOST array of n_items entries (device pointers inside).  Up to
 * 16 items share a launch.  Asynchronous on the stream. */
typedef struct heta_adam_item {
    void *table;             /* device [n_table_rows, ld_table] of dt */
    heta_dtype dt;
    int64_t ld_table;
    int32_t d;
    int64_t n_table_rows;
    float *m, *v;            /* device fp32 [n_table_rows, ld_state] */
    int64_t ld_state;
    const int64_t *ids;      /* device [n] distinct rows, or NULL for the first n rows */
    int64_t n;
    const float *grad;       /* device fp32 [n, ld_grad] */
    int64_t ld_grad;
} heta_adam_item;
heta_status heta_sparse_adam_multi(int32_t n_items, const heta_adam_item *items, float lr, float beta1, float beta2, float eps,
                                   int64_t step, void *hip_stream);

/* ---- meta-partitioning (Section 5, Algorithm 2): which relations a GPU (or machine) holds ---------
 * Host-only: works on the weighted metagraph, touches no device.  All pointers are HOST arrays.
 *   type_weight [n_types]: nodes per node type; rel_src, rel_dst, rel_weight [n_rels]: the relations
 *   (messages flow src -> dst) and their edge counts; root: the target node type; k: number of layers
 *   (depth of the metatree); p: number of partitions.
 *   metapath_ptr [n_metapaths + 1] / metapath_rels: optional user-given metapaths as relation indices
 *   listed from the root outwards (the first relation ends in `root`, each next one ends in the source
 *   type of the one before); n_metapaths = 0 (pointers may be NULL): the metatree is the tree of all
 *   walks of at most k relations from the root.
 * Steps: metatree; one sub-metatree per child of the root (root + child + descendants), weighted by
 * its node types (each once) plus its links (each per occurrence); longest-processing-time-first
 * assignment (heaviest first, equal weights by lower relation index, to the partition with the smallest
 * sum, equal sums to the lowest index); per partition the union of its sub-metatrees' relations and
 * types.  With more partitions than sub-metatrees each further partition replicates the one with the
 * largest weight per replica (replicas split the target nodes between them).
 * Outputs (caller-allocated, overwritten):
 *   *n_sub; sub_rel, sub_weight, sub_links, sub_part [capacity n_rels]: per sub-metatree the relation
 *   from the root to its child, its weight, the link part of the weight, and its partition;
 *   part_weight [p]: the assignment's sums (0 for replicas); replica_of [p]: -1 or the partition copied;
 *   rel_mask [p * n_rels], type_mask [p * n_types]: 1 where partition q holds relation i / type t.
 * HETA_ERR_INVALID_ARG for a null pointer, an index out of range, a negative weight, k < 1, p < 1 or a
 * metapath that does not follow the metagraph; HETA_ERR_UNSUPPORTED if the metatree would exceed 2^22
 * vertices. */
heta_status heta_meta_partition(int32_t n_types, const int64_t *type_weight, int32_t n_rels, const int32_t *rel_src,
                                const int32_t *rel_dst, const int64_t *rel_weight, int32_t root, int32_t k, int32_t p,
                                int32_t n_metapaths, const int32_t *metapath_ptr, const int32_t *metapath_rels,
                                int32_t *n_sub, int32_t *sub_rel, int64_t *sub_weight, int64_t *sub_links,
                                int32_t *sub_part, int64_t *part_weight, int32_t *replica_of, uint8_t *rel_mask,
                                uint8_t *type_mask);

/* ---- measurement --------------------------------------------------------------------------------
 * With profiling on (process-wide), every kernel the library launches is bracketed by two HIP
 * events on the stream it runs on.  heta_profile_read waits for the outstanding events and
 * returns one record per kernel name: launches, summed duration, and the algorithmic bytes and
 * flops of those launches (per relation and direction: E*d*sizeof(in) + 4*E + 8*rows +
 * rows*d*sizeof(out) for an aggregation; 2*n*d_in*d_out flops for a projection).
 * `out` is a HOST array of `capacity` records; *n_out receives the number of kernels seen. */
typedef struct {
    char name[48];
    int64_t launches;
    double total_ms;
    double algorithmic_bytes;
    double flops;
} heta_kernel_stat;
heta_status heta_profile_enable(int32_t on);
heta_status heta_profile_reset(void);
heta_status heta_profile_read(heta_kernel_stat *out, int32_t capacity, int32_t *n_out);
/* A plain device-to-device streaming copy of n_bytes (multiple of 16, 16-byte aligned buffers):
 * the kernel of known traffic against which hardware byte counters are scaled. */
heta_status heta_calibration_copy(void *dst, const void *src, int64_t n_bytes, void *hip_stream);
/* Matrix instructions on registers only (no memory traffic): 512 workgroups of four wavefronts, each
 * issuing 16 * iters independent 32 x 32 MFMAs of dt's kind (fp32: 32x32x2, bf16: 32x32x16).  Timing it
 * gives the rate the matrix pipes sustain at the clock the chip holds under that load, the reference
 * point beside the published peak when a projection kernel's MFMA rate is judged.  varying = 0: one
 * operand pair with zeros on one side; varying != 0: four operand pairs of mixed signs and significands taken
 * in turn, so that multipliers and accumulators see new bits with every instruction, as they do on real data
 * (the chip's power management then holds a lower clock).  sink: device, sink_elems >= 2048 floats
 * (overwritten); flops_out (host, nullable) receives the launch's flop count.  1 <= iters <= 2^24. */
heta_status heta_calibration_mfma(heta_dtype dt, int32_t varying, int64_t iters, float *sink, int64_t sink_elems,
                                  double *flops_out, void *hip_stream);

/* Message of the last failure on the calling thread (valid until that thread's next call). */
const char *heta_last_error(void);
/* "major.minor" of the library. */
const char *heta_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HETA_H */
