/*
 * gt.h -- C ABI of the MI355X (gfx950) GNN aggregation / combination library.
 *
 * The library implements the GPU hot path of GraphTensor (arXiv 2305.17469):
 *   - `Pull`, the destination-centric, feature-wise neighbour aggregation  Y = A X  over an
 *     in-edge CSR (paper: Preliminaries "Data representation"; Frontend section, the Pull
 *     primitive), and its derivative, an aggregation whose outputs live on the source vertices
 *     (paper: "Training for GNNs"), run over the transposed structure,
 *   - `Apply`, the dense combination  act(M W + b)  and its derivatives (same sections),
 *   - the kernel orchestrator's run-time choice between aggregation-first
 *     act(A X W + b) = sigma(W f(h(X)) + b)  and combination-first  sigma(f(h(W X)) + b)
 *     (paper: GNN Kernel Orchestrator, "Dynamic kernel placement" and the DKP cost model table).
 *
 * Conventions (hold for every entry point unless it says otherwise)
 *   Layout     matrices are row-major, nodes x features; `ld*` is the row stride in ELEMENTS
 *              (>= the logical width).  Rows whose stride in bytes and base address are
 *              multiples of 16 take the vectorised kernels; anything else takes a slower
 *              element-wise path with identical results up to summation order.
 *   Pointers   every data pointer is a DEVICE pointer unless marked "host".  The caller owns
 *              all device memory (inputs, outputs, workspaces); the library never allocates or
 *              frees device memory and never keeps a pointer beyond what is stated.
 *   Streams    `stream` is a hipStream_t passed as void* (NULL = the default stream).  Compute
 *              calls only enqueue work and return; gt_graph_create synchronises the stream (twice).
 *   dtype      GT_F32: fp32 storage and arithmetic.  GT_BF16: bf16 storage (round-to-nearest-
 *              even on store), fp32 accumulation.
 *   Errors     every call returns a gt_status; nothing throws, aborts or prints.  Arguments
 *              are validated on the host (null pointers, negative sizes, ld < width, workspace
 *              too small, unsupported combinations) BEFORE anything is launched; device array
 *              CONTENTS are trusted (use gt_graph_validate to check them).
 *              gt_last_error() gives a thread-local message for the last failing call.
 *   Results    no floating-point atomics anywhere: results are bit-wise reproducible from run
 *              to run for the same inputs and the same plan.
 */
#ifndef GT_H
#define GT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GT_OK = 0,
    GT_ERR_INVALID_ARG = 1,  /* null pointer, negative size, ld < width, aliasing in == out */
    GT_ERR_UNSUPPORTED = 2,  /* e.g. symmetric norm on a non-square graph, E >= 2^31 - 1024 */
    GT_ERR_WORKSPACE = 3,    /* workspace pointer null / misaligned / too small             */
    GT_ERR_HIP = 4,          /* a HIP runtime call failed (message in gt_last_error)        */
    GT_ERR_INTERNAL = 5
} gt_status;

typedef enum { GT_F32 = 0, GT_BF16 = 1 } gt_dtype;

/* Aggregation function f (paper: "Algorithm model", e.g. arithmetic mean; the `mode` string
 * of Pull).  For destination v with in-edges e = (u -> v), per-edge scalar weight w_e (1 if
 * the graph has none; the weighting function h of the paper restricted to scalars):
 *   GT_SUM      Y[v] = sum_e w_e X[u]
 *   GT_MEAN     Y[v] = (sum_e w_e X[u]) / indeg(v)           (0 for an empty row)
 *   GT_SYMNORM  Y[v] = d(v)^-1/2 sum_e w_e d(u)^-1/2 X[u],   d = in-degree of the given CSR for
 *               both ends, d^-1/2 := 0 where d = 0; square graphs (n_src == n_dst) only.
 * GT_SYMNORM is not in the paper (its GCN is mean based); it is the usual GCN normalisation. */
typedef enum { GT_SUM = 0, GT_MEAN = 1, GT_SYMNORM = 2 } gt_reduce;

/* Kernel placement (paper: "Dynamic kernel placement").  For the backward pass the value names
 * the derivative of that forward composition: GT_AGG_FIRST runs the transposed aggregation at
 * width in_dim (dM = dZ W^T, then A^T dM), GT_COMB_FIRST at width out_dim (A^T dZ, then ... W^T). */
typedef enum { GT_AUTO = 0, GT_AGG_FIRST = 1, GT_COMB_FIRST = 2 } gt_order;

typedef enum { GT_ACT_NONE = 0, GT_ACT_RELU = 1 } gt_act;

typedef struct gt_graph gt_graph; /* opaque HOST handle; borrows the caller's device arrays */

/* ------------------------------------------------------------------------------------------
 * Graph plan (once per graph / per sampled block).
 * The paper keeps the forward structure in CSR and states that CSC suits the backward pass
 * ("Training for GNNs"); it does not say how CSC is obtained.  Here it is built once per graph:
 * degrees, the transposed structure (rows by source, entries ordered by position in the given
 * CSR, i.e. a stable sort), and the degree-binned work lists that split long rows.
 * ------------------------------------------------------------------------------------------ */

/* Bytes of device workspace gt_graph_create needs (host out-pointer).  */
gt_status gt_graph_plan_size(int64_t n_dst, int64_t n_src, int64_t n_edges, int has_edge_weight,
                             size_t *ws_bytes /* host */);

/* rowptr[n_dst+1], colidx[n_edges] (source ids in [0, n_src)), edge_weight[n_edges] or NULL:
 * device, int32/fp32, borrowed until gt_graph_destroy.  ws: device, 256-byte aligned, at
 * least gt_graph_plan_size bytes, borrowed likewise (it holds the plan).  Enqueues the plan
 * kernels on `stream` and synchronises it twice: once to read back the work-list sizes, once
 * before returning, so that the finished plan may be used from any stream.
 * Errors: INVALID_ARG (null/negative), UNSUPPORTED (n_edges or n_* >= 2^31 - 1024), WORKSPACE, HIP. */
gt_status gt_graph_create(gt_graph **g /* host out */, int64_t n_dst, int64_t n_src, int64_t n_edges,
                          const int32_t *rowptr, const int32_t *colidx, const float *edge_weight,
                          void *ws, size_t ws_bytes, void *stream);

/* Frees the host handle only. */
gt_status gt_graph_destroy(gt_graph *g);

/* Device pointers into the plan (any out-pointer may be NULL): in_deg[n_dst], out_deg[n_src],
 * rowptr_t[n_src+1], colidx_t[n_edges] (destination of each transposed entry), perm[n_edges]
 * (position of that entry in the given CSR).  All int32 and exactly defined (bit-exact). */
gt_status gt_graph_outputs(const gt_graph *g, const int32_t **in_deg, const int32_t **out_deg,
                           const int32_t **rowptr_t, const int32_t **colidx_t, const int32_t **perm);

/* Host-side sizes of the plan: n_dst, n_src, n_edges, and the number of work items / split
 * rows of the forward and transposed schedules (any out-pointer may be NULL). */
gt_status gt_graph_info(const gt_graph *g, int64_t *n_dst, int64_t *n_src, int64_t *n_edges,
                        int64_t *fwd_items, int64_t *fwd_split_rows, int64_t *bwd_items,
                        int64_t *bwd_split_rows);

/* Debug check of the borrowed arrays: counts rowptr[0] != 0, rowptr[n_dst] != n_edges,
 * decreasing rowptr, colidx outside [0, n_src).  Synchronises; *n_violations is a host int64. */
gt_status gt_graph_validate(const gt_graph *g, int64_t *n_violations /* host */, void *stream);

/* ------------------------------------------------------------------------------------------
 * Aggregation (Pull) and its derivative.
 * ------------------------------------------------------------------------------------------ */

/* Bytes of scratch an aggregation at width F needs on this graph (fp32 partial rows of the
 * split long rows; 0 if no row is split).  Covers both directions. */
gt_status gt_aggregate_ws_size(const gt_graph *g, int64_t F, size_t *ws_bytes /* host */);

/* Y[n_dst, F] = A X,  X[n_src, F];  see gt_reduce.  X and Y must not overlap.  ws: device
 * scratch of at least gt_aggregate_ws_size bytes (may be NULL when that is 0), 256-byte aligned;
 * its contents are overwritten.  Errors: INVALID_ARG, UNSUPPORTED (SYMNORM on a non-square
 * graph), WORKSPACE.  n_dst == 0 or F == 0 is a valid no-op; empty rows give zeros. */
gt_status gt_aggregate_fwd(const gt_graph *g, gt_reduce reduce, gt_dtype dtype, int64_t F,
                           const void *X, int64_t ldx, void *Y, int64_t ldy,
                           void *ws, size_t ws_bytes, void *stream);

/* dX[n_src, F] = A^T dY,  dY[n_dst, F]: the derivative of gt_aggregate_fwd with the same
 * per-edge coefficients (edge weights are constants: no gradient is produced for them). */
gt_status gt_aggregate_bwd(const gt_graph *g, gt_reduce reduce, gt_dtype dtype, int64_t F,
                           const void *dY, int64_t lddy, void *dX, int64_t lddx,
                           void *ws, size_t ws_bytes, void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): gt_aggregate_fwd with the scratch for the partial
 * rows of split long rows taken from a fixed array inside the library (32 MiB per GPU, held from
 * library load until the process ends) instead of a caller workspace.  Same arguments, checks,
 * kernels and results (bit for bit) as gt_aggregate_fwd.  Calls no hipMalloc / hipFree or other
 * allocating routine and records no kernel-timing events.  If the graph's partial rows at width
 * F need more than gt_aggregate_static_capacity() bytes (compare gt_aggregate_ws_size), returns
 * GT_ERR_WORKSPACE and launches nothing.  The GPU that is current at the call must be the one
 * that holds the graph and the tensors.  All calls on one GPU share the one array: calls that
 * may overlap in time on the same GPU (different streams or threads) race on it and must be
 * serialised by the caller; nothing in it needs to be cleared between calls. */
gt_status gt_aggregate_static_capacity(size_t *bytes /* host */);
gt_status gt_aggregate_fwd_static(const gt_graph *g, gt_reduce reduce, gt_dtype dtype, int64_t F,
                                  const void *X, int64_t ldx, void *Y, int64_t ldy, void *stream);

/* Fused aggregation-first forward for inference,  Y[n_dst, out_dim] = act( (A X) W + b ):  the
 * aggregated row of a destination stays on chip (paper: Frontend section, Pull accumulates a
 * destination's row on chip and writes it once) and is handed straight to the combination's
 * matrix instructions (Apply); A X is never written to memory, so no backward call can follow.
 * X[n_src, in_dim] (ldx; rows 16-byte aligned: otherwise GT_ERR_UNSUPPORTED), W[in_dim, out_dim]
 * dense (row stride out_dim), b[out_dim] fp32 or NULL, all data in `dtype`.  Shapes: in_dim <= 256
 * (bf16) / 128 (fp32), out_dim <= 256, and weights plus row tiles within the 160 KB of LDS
 * (gt_aggregate_combine_supported tells; GT_ERR_UNSUPPORTED otherwise).  ws as for gt_aggregate_fwd
 * at width in_dim (partial rows of split long rows).  Same results as gt_aggregate_fwd followed by
 * gt_combine up to the summation order inside the matrix instructions. */
gt_status gt_aggregate_combine_supported(gt_dtype dtype, int64_t in_dim, int64_t out_dim, int *yes /* host */);
gt_status gt_aggregate_combine_fwd(const gt_graph *g, gt_reduce reduce, gt_dtype dtype, int64_t in_dim,
                                   int64_t out_dim, const void *X, int64_t ldx, const void *W, const float *b,
                                   gt_act act, void *Y, int64_t ldy, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * Edge weighting: NeighborApply (the edge-weight function g of the source and destination
 * embeddings per edge, i.e. SDDMM) and Pull with per-call edge weights (the function h that
 * transforms the source embedding with g's output before the aggregation f); paper:
 * Preliminaries "edge weighting", "Training for GNNs" (g' is applied to both ends), Frontend
 * section (NeighborApply, Pull, the NGCF listing).  Edge e = (u -> v) is position e of the CSR the
 * plan was built from; the plan must have been built WITHOUT static edge weights (UNSUPPORTED
 * otherwise).  Xs[n_src, F], Xd[n_dst, F], Y / dY[n_dst, F], dXs[n_src, F], dXd[n_dst, F] in `dtype`.
 * Scalar edge data (GT_G_DOT, GT_H_SCALE) is float[E]; vector edge data is [E, F] in `dtype`
 * with row stride ldw.  ws as for gt_aggregate_fwd (gt_aggregate_ws_size(F)).
 *   g: GT_G_DOT  w_e = <Xs[u], Xd[v]>,   GT_G_MUL  w_e = Xs[u] (.) Xd[v]
 *   h: GT_H_SCALE  w_e * Xs[u],   GT_H_ADD  Xs[u] + w_e,   GT_H_MUL  Xs[u] (.) w_e
 *   f: GT_SUM or GT_MEAN over the in-edges of v (GT_SYMNORM: UNSUPPORTED).
 * ------------------------------------------------------------------------------------------ */
typedef enum { GT_G_DOT = 0, GT_G_MUL = 1 } gt_edge_fn;
typedef enum { GT_H_SCALE = 0, GT_H_ADD = 1, GT_H_MUL = 2 } gt_weight_fn;

/* W_e = g(Xs[u], Xd[v]) for every edge. */
gt_status gt_neighbor_apply_fwd(const gt_graph *g, gt_edge_fn fn, gt_dtype dtype, int64_t F,
                                const void *Xs, int64_t ldxs, const void *Xd, int64_t ldxd,
                                void *W, int64_t ldw, void *stream);

/* dXs[u] = sum over out-edges, dXd[v] = sum over in-edges of the derivative of g for upstream dW
 * (shape of W).  Both outputs are overwritten. */
gt_status gt_neighbor_apply_bwd(const gt_graph *g, gt_edge_fn fn, gt_dtype dtype, int64_t F,
                                const void *dW, int64_t lddw, const void *Xs, int64_t ldxs,
                                const void *Xd, int64_t ldxd, void *dXs, int64_t lddxs,
                                void *dXd, int64_t lddxd, void *ws, size_t ws_bytes, void *stream);

/* Y[v] = f_{e in in(v)} h(Xs[u], W_e). */
gt_status gt_pull_fwd(const gt_graph *g, gt_reduce reduce, gt_weight_fn h, gt_dtype dtype, int64_t F,
                      const void *Xs, int64_t ldxs, const void *W, int64_t ldw, void *Y, int64_t ldy,
                      void *ws, size_t ws_bytes, void *stream);

/* dXs[n_src, F] and dW (shape of W) for upstream dY; both overwritten. */
gt_status gt_pull_bwd(const gt_graph *g, gt_reduce reduce, gt_weight_fn h, gt_dtype dtype, int64_t F,
                      const void *dY, int64_t lddy, const void *Xs, int64_t ldxs,
                      const void *W, int64_t ldw, void *dXs, int64_t lddxs, void *dW, int64_t lddw,
                      void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * Combination (Apply): C[M,N] = act(op(A) op(B) + bias), op(A) is M x K, op(B) is K x N.
 *   transA = 0: A stored M x K (lda >= K);  transA = 1: A stored K x M (lda >= M).
 *   transB = 0: B stored K x N (ldb >= N);  transB = 1: B stored N x K (ldb >= K).
 * A and B have type `dtype`; C has type `c_dtype` (fp32 accumulation in MFMA either way; fp32
 * data uses fp32 MFMA, bf16 data bf16 MFMA).  bias[N] fp32 or NULL.  transA = 1 is the weight
 * gradient shape (reduction over the long node dimension): it is split over workgroups and
 * summed in a fixed order from `ws` (size from gt_combine_ws_size; 0 otherwise).
 * ------------------------------------------------------------------------------------------ */
gt_status gt_combine_ws_size(gt_dtype dtype, int transA, int transB, int64_t M, int64_t N, int64_t K,
                             size_t *ws_bytes /* host */);

gt_status gt_combine(gt_dtype dtype, int transA, int transB, int64_t M, int64_t N, int64_t K,
                     const void *A, int64_t lda, const void *B, int64_t ldb,
                     const float *bias, gt_act act, void *C, int64_t ldc, gt_dtype c_dtype,
                     void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * One GNN layer with dynamic kernel placement:
 *   H'[n_dst, out_dim] = act( A X W  (+ X[0:n_dst] W_root)  + b ),   X[n_src, in_dim].
 * has_root = 1 adds the root (self) linear of a GraphSAGE-style layer: the destinations are the
 * first n_dst source ids of the block.  need_dx = 0 marks the first layer of a model: only
 * parameter gradients are wanted, so an aggregation-first backward needs no transposed
 * aggregation at all (paper: cost-model paragraph on the first GNN layer).
 * ------------------------------------------------------------------------------------------ */
typedef struct {
    gt_reduce reduce;
    gt_dtype dtype;
    gt_act act;
    int64_t in_dim, out_dim;
    int has_root;
    int need_dx;
    /* The activation's derivative folded into the kernel that produces the gradient (both 0 = off;
     * they matter to gt_layer_bwd only).  The input X of a layer is the output of the layer below;
     * if that output went through a ReLU, dL/d(its pre-activation) = dX (.) [X > 0].
     *   in_act = GT_ACT_RELU: gt_layer_bwd writes dX already multiplied by [X > 0], as the rows are
     *            stored (no extra pass over dX).
     *   dy_is_dz != 0: the dY handed to gt_layer_bwd already carries this layer's own activation
     *            derivative (the layer above produced it with in_act set), so it is used as dZ as it
     *            is; Y is not read then and may be NULL. */
    gt_act in_act;
    int dy_is_dz;
    /* pad_writable != 0: the rows of the caller's output tensors (Y of gt_layer_fwd, dX of gt_layer_bwd)
     * are padded (ld > width) and the padding belongs to nobody else: the library may store zeros in the
     * columns from the width up to the next multiple of 16 bytes, where they lie below ld.  A row end
     * written in 2- or 4-byte pieces leaves a hole in its 32-byte sector, which the memory system has to
     * read back and merge; with whole 16-byte stores it does not (2^21 rows of 47 bf16 columns: the
     * aggregation that writes them 0.98 -> 0.92 ms, the product 0.33 -> 0.26 ms).  0 = never touch a
     * byte outside the logical tensor. */
    int pad_writable;
} gt_layer_desc;

/* Coefficients of the kernel-time model behind the placement decision (paper: "DKP cost model
 * and parameters"): combination of `rows` rows takes rows*(alpha*in*out + beta*width) and an
 * aggregation at width F takes F*(gamma*n_edge + delta*n_out); separate sets for the forward
 * (FWP) and backward (BWP) pass.  Differences of these times are exactly the four "benefit"
 * formulas of the paper's table.  Units: seconds.  The paper's own constants were fitted on
 * another GPU and are NOT the defaults; gt_calibrate refits them on this device. */
typedef struct {
    double alpha_fwd, beta_fwd, gamma_fwd, delta_fwd;
    double alpha_bwd, beta_bwd, gamma_bwd, delta_bwd;
    /* One addition to the paper's model: no aggregation launch is modelled faster than this many
     * seconds (launch plus the chain of dependent loads of one work item), so that on a graph of a
     * few thousand vertices a narrower aggregation does not count as a faster one.  Fitted by
     * gt_calibrate like the other coefficients (the time of an aggregation on a tiny graph); 0 = none. */
    double aggr_floor;
} gt_cost_coeffs;

gt_status gt_cost_get(gt_cost_coeffs *c /* host */);          /* the fp32 set */
gt_status gt_cost_set(const gt_cost_coeffs *c /* host */);    /* installs c for every data type */

/* One coefficient set per data type (the paper fits one set per system; bf16 kernels move half
 * the bytes and use a faster matrix pipe, so their times scale differently from fp32 ones).
 * gt_layer_decide and the GT_AUTO orders use the set of the layer's dtype.  Coefficients must be
 * finite and >= 0 (GT_ERR_INVALID_ARG otherwise).  The sets are process-wide and not locked:
 * set or calibrate them before layers are decided on other threads. */
gt_status gt_cost_get_dtype(gt_dtype dtype, gt_cost_coeffs *c /* host */);
gt_status gt_cost_set_dtype(gt_dtype dtype, const gt_cost_coeffs *c /* host */);

/* The four benefit values of the paper's cost-model table for the given sizes and coefficients
 * (pure host arithmetic): aggr-first FWP/BWP, comb-first FWP/BWP.  first_layer != 0 uses n_src
 * as the BWP reduction factor of aggr-first, as the paper prescribes for the first layer. */
gt_status gt_cost_benefits(const gt_cost_coeffs *c, int64_t n_src, int64_t n_dst, int64_t n_edge,
                           int64_t n_feat, int64_t n_hid, int first_layer,
                           double *aggr_fwd, double *aggr_bwd, double *comb_fwd, double *comb_bwd);

/* Placement for this layer on this graph (pure host, deterministic): comb-first iff its benefit
 * is strictly larger; a tie keeps the original aggregation-first order.  With need_dx = 0 the
 * forward and backward are decided together (the backward can only skip the aggregation if the
 * forward ran aggregation-first and saved A X). */
gt_status gt_layer_decide(const gt_graph *g, const gt_layer_desc *d, gt_order *fwd, gt_order *bwd);

/* Device bytes for `saved` (activations the backward needs, written by gt_layer_fwd) and for
 * `scratch` (temporaries of either call), for any order. */
gt_status gt_layer_ws_size(const gt_graph *g, const gt_layer_desc *d,
                           size_t *saved_bytes /* host */, size_t *scratch_bytes /* host */);

/* X[n_src,in_dim] (ldx), W[in_dim,out_dim] and W_root (dense, ld = out_dim; NULL iff !has_root)
 * in d->dtype, b[out_dim] fp32 or NULL, Y[n_dst,out_dim] (ldy) in d->dtype.  `req` forces an
 * order or GT_AUTO; *used (host, may be NULL) receives the order that ran.
 * saved / scratch: device, 256-byte aligned, at least the sizes gt_layer_ws_size reports
 * (saved_bytes / scratch_bytes are the callers' buffer sizes; GT_ERR_WORKSPACE when too small,
 * before anything is launched).  `saved` is written only by an aggregation-first forward.
 * saved == NULL (saved_bytes 0) makes the call forward-only (inference): no gt_layer_bwd may
 * follow; A X is then a temporary in `scratch`, or is never written at all where the fused kernel
 * of gt_aggregate_combine_fwd applies and is the faster path.  X and Y must not overlap
 * (GT_ERR_INVALID_ARG). */
gt_status gt_layer_fwd(const gt_graph *g, const gt_layer_desc *d, gt_order req,
                       const void *X, int64_t ldx, const void *W, const void *W_root, const float *b,
                       void *Y, int64_t ldy, void *saved, size_t saved_bytes,
                       void *scratch, size_t scratch_bytes, gt_order *used, void *stream);

/* dY[n_dst,out_dim] in d->dtype; X, W, W_root, Y, saved as given to / produced by gt_layer_fwd
 * with forward order `fwd_used`.  Outputs: dX[n_src,in_dim] in d->dtype (NULL iff !need_dx),
 * dW[in_dim,out_dim], dW_root (NULL iff !has_root), db[out_dim] (may be NULL): always fp32,
 * overwritten (not accumulated).  `req` forces the backward order or GT_AUTO.  saved / scratch
 * and their sizes as for gt_layer_fwd (`saved` is read only after an aggregation-first forward);
 * dX must not overlap dY or X. */
gt_status gt_layer_bwd(const gt_graph *g, const gt_layer_desc *d, gt_order fwd_used, gt_order req,
                       const void *dY, int64_t lddy, const void *X, int64_t ldx,
                       const void *W, const void *W_root, const void *Y, int64_t ldy,
                       const void *saved, size_t saved_bytes, void *scratch, size_t scratch_bytes,
                       void *dX, int64_t lddx, float *dW, float *dW_root, float *db,
                       gt_order *used, void *stream);

/* Refit the cost coefficients by least squares from kernel times measured on this device
 * (paper: coefficients are fitted from measured kernel times at the start of training).  Runs
 * synthetic aggregations and combinations inside `ws` (device, >= gt_calibrate_ws_size bytes);
 * synchronises.  gt_calibrate_dtype fits and installs the set of one data type (as by
 * gt_cost_set_dtype) and returns it in *fitted; gt_calibrate does so for bf16 and then fp32 and
 * returns the fp32 set. */
gt_status gt_calibrate_ws_size(size_t *ws_bytes /* host */);
gt_status gt_calibrate(void *ws, size_t ws_bytes, gt_cost_coeffs *fitted /* host, may be NULL */, void *stream);
gt_status gt_calibrate_dtype(gt_dtype dtype, void *ws, size_t ws_bytes, gt_cost_coeffs *fitted /* host, may be NULL */,
                             void *stream);

/* ------------------------------------------------------------------------------------------
 * Batch preparation on the GPU: neighbour sampling (S), renumbering (R) and embedding lookup (K)
 * (paper: Preliminaries, "Preprocessing for GNNs"; Service-wide tensor scheduler,
 * "High-performance preprocessing").  The paper runs S, R and K on host threads, because graph
 * and embedding table live in host memory, and adds T, the transfer to the GPU.  Here graph and
 * table are resident in device memory: S, R and K are kernels on the caller's stream (so a
 * batch can be prepared on one stream while the previous one trains on another) and T is gone.
 *
 * One subgraph per GNN layer, the layer nearest the seeds first: S on the seeds, R, then S on
 * R's source list for the next layer outwards, R again, ..., and K on the outermost source list.
 *
 * The random choice ("unique random" in the paper, not specified further) is a keyed
 * pseudo-random permutation pi of the positions 0..d-1 of a destination's in-neighbour list:
 *   mix32(x): x ^= x>>16; x *= 0x7feb352d; x ^= x>>15; x *= 0x846ca68b; x ^= x>>16   (mod 2^32)
 *   row key  rk = mix32(mix32(seed + 0x9E3779B9 * stream_id) ^ v),   v = global destination id
 *   d <= 64: position j has key mix32(rk + 0x9E3779B9 * (j + 1)); pi orders positions by key
 *   d >  64: 6-round balanced Feistel network on 2h bits (h = ceil(bitlength(d-1) / 2), round
 *            r maps (L, R) to (R, L ^ (mix32(R ^ mix32(rk + 0x9E3779B9 * (r + 1))) & (2^h-1)))),
 *            re-applied until the value is < d
 * A destination with d <= fanout keeps its whole list in list order; otherwise its picks are
 * colidx[rowptr[v] + pi(t)], t = 0..fanout-1, in that order.  The result depends on
 * (seed, stream_id, v) only, not on the rest of the batch, and is bit-wise reproducible.
 * ------------------------------------------------------------------------------------------ */

/* S.  rowptr[n_vertices + 1], colidx: in-edge CSR of the WHOLE graph, global ids.  dst[n_dst]:
 * the layer's destinations (global ids; an id outside [0, n_vertices) yields an empty row).
 * out_rowptr[n_dst + 1]: offsets of the sampled rows; out_nbr: the picked global ids, capacity
 * n_dst * fanout entries (< 2^31).  ws: >= gt_sample_ws_size bytes, 256-byte aligned. */
gt_status gt_sample_ws_size(int64_t n_dst, size_t *ws_bytes /* host */);
gt_status gt_sample_neighbors(const int32_t *rowptr, const int32_t *colidx, int64_t n_vertices,
                              const int32_t *dst, int64_t n_dst, int32_t fanout, uint32_t seed,
                              uint32_t stream_id, int32_t *out_rowptr, int32_t *out_nbr,
                              void *ws, size_t ws_bytes, void *stream);

/* R.  The table of sampled vertices: walking dst[0..n_dst) and then picked[0..n_picked) in
 * order, an id met for the first time receives the next new id, counted from 0.  dst must hold
 * distinct ids (then destination i has new id i); all ids must lie in [0, n_vertices).
 *   src_global[n_dst + n_picked] (capacity): global id of every new id, first n_src entries;
 *   colidx_local[n_picked]: picked[] rewritten in new ids (same order);
 *   counts[2] (device): n_src, and the number of distinct ids among dst (== n_dst iff the
 *   precondition holds; nothing else is guaranteed when it does not).
 * Implemented as a stable radix sort of (id, position) and two scans: no hash table, no
 * atomics, so the first-met order is exact.  n_dst + n_picked < 2^31. */
gt_status gt_reindex_ws_size(int64_t n_dst, int64_t n_picked, size_t *ws_bytes /* host */);
gt_status gt_reindex(const int32_t *dst, int64_t n_dst, const int32_t *picked, int64_t n_picked,
                     int64_t n_vertices, int32_t *src_global, int32_t *colidx_local,
                     int32_t *counts, void *ws, size_t ws_bytes, void *stream);

/* K.  out[i, 0:F] = table[ids[i], 0:F] for i < n; an id outside [0, n_rows) yields a row of
 * zeros.  Only the F logical columns of `out` are written. */
gt_status gt_lookup(gt_dtype dtype, const void *table, int64_t n_rows, int64_t ld,
                    const int32_t *ids, int64_t n, int64_t F, void *out, int64_t ldo, void *stream);

/* ------------------------------------------------------------------------------------------
 * Optional per-kernel timing (the paper reports GPU kernel time measured with a profiler; this
 * gives the same quantity from inside a timed region).  While enabled, every aggregation
 * gather kernel and every combination kernel launched by this library is bracketed by two HIP
 * events on its own stream.  Host-side state, not thread-safe; off by default.
 *   kind: 0 aggregation (given CSR), 1 aggregation (transposed), 2 combination, 3 fused
 *   aggregation + combination (width = in_dim)
 *   width: feature width F (aggregation) or N (combination); rows: output rows;
 *   work: edges gathered (aggregation) or M*N*K (combination); ms: kernel duration.
 * gt_trace_get synchronises on the record's end event.
 * ------------------------------------------------------------------------------------------ */
gt_status gt_trace_enable(int on);
gt_status gt_trace_reset(void);
gt_status gt_trace_count(int64_t *n /* host */);
gt_status gt_trace_get(int64_t i, int *kind, int64_t *width, int64_t *rows, int64_t *work, double *ms);
/* Which instance of the aggregation kernel record i timed: V elements per lane and load, G lanes
 * per work item, NP column tiles per lane, U row loads in flight, and whether it applies an output
 * mask (all 0 for a combination record).  Together with the data type these are the kernel's
 * template arguments, i.e. its name in a profiler's kernel list. */
gt_status gt_trace_get_variant(int64_t i, int *V, int *G, int *NP, int *U, int *masked);

const char *gt_status_string(gt_status s);
const char *gt_last_error(void);
const char *gt_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GT_H */
