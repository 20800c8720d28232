/*
 * gsr.h - C ABI of the MI355X (gfx950) GSR-GNN training-step library.
 *
 * One training step of the deep grouped-reversible GNN stack of arxiv 2603.27156
 * ("GSR-GNN"): forward, inverse recomputation in place of stored activations, backward.
 *
 *   layer (Section 3, eq. (6)):   Y_0 = sum_{j=2..C} X_j,   Y_i = f_i(Y_{i-1}, A) + X_i,  i = 1..C
 *   inverse (Section 3, eq. (7)): X_i = Y_i - f_i(Y_{i-1}, A),  i = C..1
 *   block (Section 4.1, eq. (10)): f_i(Z, A) = ( A * scatter(GS(Z, k)) ) * W_i
 *   GS (Section 4.1):             per row, the k largest entries by signed value -> (V, I)
 *
 * Conventions
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *     ordinary host memory.  The library never frees or reallocates caller memory.
 *   - gsr_graph_create / gsr_graph_destroy own the device memory of the graph they build (the CSR, its split
 *     plan, tile counters, and the scratch of gsr_spmm and gsr_graph_normalize).  No other call allocates device
 *     memory; scratch comes from the caller's `workspace`.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = default stream)
 *     and is asynchronous unless stated.  Calls on one graph / workspace must be ordered:
 *     a graph holds the tile counters its kernels draw work from and the first-pass sums of
 *     its split rows, so two calls that use the same graph must not overlap on different
 *     streams (build one graph per stream for that).  The layer and step calls only launch
 *     kernels (unless "profile" is set), so they can be captured into a HIP graph and replayed.
 *   - Every call returns a gsr_status_t and never throws or aborts.  gsr_last_error()
 *     gives a thread-local message for the last failure on the calling thread.
 *   - Weights W_i are dg x dg, row-major, "in -> out":  O[n][o] = sum_m H[n][m] W_i[m][o].
 *   - Results are deterministic: no floating-point atomics are used anywhere.
 */
#ifndef GSR_H_
#define GSR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum gsr_status {
    GSR_OK = 0,
    GSR_ERR_INVALID_ARG = 1,         /* null pointer, negative size, inconsistent sizes */
    GSR_ERR_BAD_CSR = 2,             /* non-monotone row pointers, column out of range */
    GSR_ERR_UNSUPPORTED = 3,         /* C < 2, k < 1, k > D/C, D % C != 0, D/C not among those built, dtype */
    GSR_ERR_WORKSPACE_TOO_SMALL = 4, /* workspace_bytes below gsr_workspace_size() */
    GSR_ERR_HIP = 5                  /* a HIP runtime call failed (message has the HIP error) */
} gsr_status_t;

/* Storage type of activation planes, gradient planes and compressed values.  All arithmetic
 * accumulates in float32; weights and weight gradients are always float32. */
typedef enum gsr_dtype { GSR_F32 = 0, GSR_BF16 = 1 } gsr_dtype_t;

/* Scale applied to the k retained values of a row inside a block.  NONE is the operator as
 * Section 4.1 defines it.  RMS divides the kept values by sqrt(mean_c Z[n][c]^2 + eps) of
 * the whole row (no learnable parameters); the selection itself always uses the raw row. */
typedef enum gsr_norm { GSR_NORM_NONE = 0, GSR_NORM_RMS = 1 } gsr_norm_t;

/* Memory layout of an N x D plane handed to the layer / step calls.
 * ROW_MAJOR:     element (n, group i, c) at  n*D + i*(D/C) + c      (Split/Concat of eq. (1)
 *                and Algorithm 1 are then plain column slices).
 * GROUP_PLANAR:  element (n, group i, c) at  i*N*(D/C) + n*(D/C) + c  (what gsr_step uses
 *                internally: every per-group pass is one contiguous stream). */
typedef enum gsr_layout { GSR_LAYOUT_ROW_MAJOR = 0, GSR_LAYOUT_GROUP_PLANAR = 1 } gsr_layout_t;

/* gsr_graph_create flags */
#define GSR_GRAPH_SYMMETRISE 1u      /* store A + A^T (pattern union)                      */
#define GSR_GRAPH_ADD_SELF_LOOPS 2u  /* exactly one diagonal entry per row                 */
#define GSR_GRAPH_GCN_NORM 4u        /* values = d_i^-1/2 d_j^-1/2, d = stored row length  */
#define GSR_GRAPH_ROWPTR_I64 8u      /* `rowptr` points at int64 (else int32)              */

typedef enum gsr_adj_norm { GSR_ADJ_UNIT = 0, GSR_ADJ_GCN_SYM = 1 } gsr_adj_norm_t;

typedef struct gsr_graph gsr_graph_t; /* opaque */

/* Limits of this build (anything beyond is refused with GSR_ERR_UNSUPPORTED, never computed wrongly):
 *   N < 2^31 nodes; fewer than 2^31 stored entries after symmetrisation and self-loops (device row pointers are
 *   32-bit; the input row pointers may be 64-bit);  N * k < 2^32 (32-bit offsets into the compressed values);
 *   2 <= C <= 8;  D/C in {32, 64, 128, 192, 256};  gsr_step: D <= 512 (the scalar head).
 *   D/C above 64 (the paper's own models: hidden 256 or 384 in two groups, Section 5) runs as D/C / 64 column blocks of
 *   64 through the same kernels, (D/C / 64)^2 launches per block, with GS over the whole row; it takes
 *   save_indices 0 or 1. */
typedef struct gsr_config {
    int64_t n;      /* nodes N */
    int32_t d;      /* feature width D */
    int32_t c;      /* groups C (2..8); D/C must be 32, 64, 128, 192 or 256 */
    int32_t l;      /* layers L (gsr_step only) */
    int32_t k;      /* retained elements per row per group, 1 <= k <= D/C */
    int32_t dtype;  /* gsr_dtype_t */
    int32_t norm;   /* gsr_norm_t */
    float eps;      /* RMS epsilon */
    int32_t layout; /* gsr_layout_t of caller-side N x D planes */
    int32_t save_indices; /* gsr_step only.  0: GS is applied again to the rebuilt activations during
                             the inverse and nothing is kept per layer (workspace independent of L).
                             1: the column set every block selected in the forward sweep is kept
                             (Section 4.2: selective save of the indices, O(L N k) bits) and reused by
                             the inverse, which is then continuous in its input; the workspace grows
                             by (L+1) * C * N * (D/C)/8 bytes.
                             2: as 1, but only for the rows that selected at a near-tie: with v_k the k-th
                             and v_(k+1) the (k+1)-th largest value of a row, the row's column set is kept
                             iff v_k - v_(k+1) <= tie_tol * max|row| (float32 arithmetic; exact ties always
                             are).  Every other row selects again on its rebuilt values, which gives the
                             same set as long as the rebuilt row is off by less than half its gap.  The
                             workspace grows by (L+1) * C * (2048 + tie_capacity * (4 + (D/C)/8)) bytes. */
    float tie_tol;        /* save_indices == 2: see above; >= 0.  Rounding of the inverse sweep grows with depth
                             (measured on 1M nodes, D/C = 64, float32: rebuilt input off by 2e-4 of its range at
                             L = 448): 2^-12 covers that depth, deeper stacks need more. */
    int32_t tie_capacity; /* save_indices == 2: rows that can be kept per block and layer; 0: N/32 + 1024.  Kept as
                             sixteen sub-lists of tie_capacity / 16 places (rounded up), tile t appending to sub-list
                             t mod 16, each with its own counter (so a block whose near-tie rows crowd into few
                             tiles keeps fewer than tie_capacity of them).
                             Rows beyond it are not kept and select again (gsr_step_tie_stats counts them); which
                             rows of a block those are depends on the order the waves append in, so results are
                             bit-reproducible between runs only while nothing is dropped. */
} gsr_config_t;

const char* gsr_last_error(void);
const char* gsr_version(void);

/* Process-wide tunables, read by the next gsr_graph_create:
 *   "hub_threshold"   rows with more stored entries than this are reduced in two passes (Section 2 notes nets
 *                     with more than 8,000 neighbours); 0, the default: 512; 64 or 16 on graphs with fewer than
 *                     four / two 16-row tiles per resident wave; 1 on graphs whose mean row has 64 stored entries or
 *                     more (every row of two entries or more then goes through the first pass)
 *   "hub_chunk"       neighbours per first-pass partial sum; 0, the default: 64, or 512 on graphs of long rows
 *   "hub_values"      how the first pass sums float32 records (layer and step calls): 1 = a lane per record value,
 *                     through a byte per value naming its column that a small kernel writes from the masks first;
 *                     2 = a lane per group of columns, as the tile kernels do; 0, the default: 1 on graphs whose mean
 *                     row has 64 stored entries or more, while 2 k <= D/C (groups of 128 or 192 columns: one such
 *                     pass for all their column blocks; of 256: a pass per block of 64 while 2 k <= 64).  Read when
 *                     a graph is created
 *   "max_workgroups"  workgroups of the persistent kernels, multiple of 8 (0: as many as stay resident, at most 4 per CU)
 *   "profile"         bit mask of kernel classes to time (see gsr_profile_read); read at once */
gsr_status_t gsr_set_option(const char* key, int64_t value);

/* Measurement aid.  gsr_set_option("profile", mask) makes the layer / step calls bracket every
 * launch of kernel class i (bit i of mask) with HIP events on the caller's stream.
 * gsr_profile_read waits for the recorded events and returns the summed duration and number
 * of launches of one class since the last gsr_profile_reset.  Classes: 0 block forward,
 * 1 block inverse, 2 block inverse + weight gradient, 3 data gradient, 4 group sum / record,
 * 5 hub first pass, 6 dW reduction (on large graphs it is part of class 3), 7 head, 8 layout copy, 9 records of
 * near-tie rows written again (save_indices == 2), 10 weight gradient dW_i = H^T dY_i (class 2 is no longer launched:
 * the inverse of the backward runs as class 1).  Not thread-safe. */
gsr_status_t gsr_profile_read(int32_t kernel_class, double* total_ms, int64_t* launches);
gsr_status_t gsr_profile_reset(void);
const char* gsr_profile_class_name(int32_t kernel_class);

/* ---- graph: adjacency A of Section 3 (forward aggregates over G, backward over G^T) ----
 *
 * Builds the device CSR used by every other call from a host CSR of n rows and nnz entries
 * (`rowptr`: n+1 int32 or int64; `colidx`: nnz int32 in [0,n), any order, duplicates
 * allowed).  With SYMMETRISE / ADD_SELF_LOOPS the pattern is transformed first (duplicates
 * merged, columns ascending).  Values: GCN_NORM computes d_i^-1/2 d_j^-1/2 on the device with
 * the fixed float32 recipe  dinv = 1.0f/sqrtf((float)deg), a_ij = dinv_i*dinv_j; otherwise
 * `vals` (host, nnz floats, entries of duplicate positions are summed) or 1.0 when NULL.
 * The transpose needed by the backward pass is built too unless the result is symmetric.
 * Synchronous.  *out is owned by the caller until gsr_graph_destroy. */
gsr_status_t gsr_graph_create(gsr_graph_t** out, int64_t n, int64_t nnz, const void* rowptr,
                              const int32_t* colidx, const float* vals, uint32_t flags, void* stream);

/* Recompute the stored values on the device: all ones, or the GCN symmetric normalisation of
 * the stored pattern as defined above.  Asynchronous on `stream`: only launches kernels (d^-1/2 passes through a
 * buffer the graph owns, so two such calls on one graph must not overlap). */
gsr_status_t gsr_graph_normalize(gsr_graph_t* g, int32_t mode /* gsr_adj_norm_t */, void* stream);

/* Sizes of the stored matrix.  Any output pointer may be NULL.  n_hub_rows = rows whose
 * length exceeds the split threshold and are reduced in two deterministic passes. */
gsr_status_t gsr_graph_info(const gsr_graph_t* g, int64_t* n, int64_t* nnz, int64_t* max_degree,
                            int64_t* n_hub_rows);

/* Copy the stored CSR to host arrays (n+1 int64, nnz int32, nnz float).  Synchronous.
 * Any output pointer may be NULL. */
gsr_status_t gsr_graph_export(const gsr_graph_t* g, int64_t* rowptr, int32_t* colidx, float* vals);

gsr_status_t gsr_graph_destroy(gsr_graph_t* g);

/* ---- operators exposed as the paper defines them ----
 *
 * GS(X, k) -> (V, I), Section 4.1.  x: device, n rows of dg values of `dtype`, row stride ld
 * elements; dg in [1, 256].  vals_out: device n*k of `dtype`; idx_out: device n*k int32, slots
 * in ascending column order.  Largest by signed value; ties to the lowest column; -0 == +0;
 * inputs must be finite.  norm/eps as in gsr_norm_t (V is the scaled value). */
gsr_status_t gsr_group_sparse(const void* x, int64_t n, int32_t dg, int64_t ld, int32_t k, int32_t dtype,
                              int32_t norm, float eps, void* vals_out, int32_t* idx_out, void* stream);

/* Y = A X (transpose = 0) or A^T X (transpose = 1) for dense float32 X: device n x width, row
 * strides ldx / ldy elements.  The plain neighbour aggregation of Section 3, eq. (2).
 * Widths 16, 32 and 64 with 4- / 8- / 16-byte aligned rows take the tiled path, which keeps the
 * first-pass sums of rows longer than "hub_threshold" in a buffer owned by the graph: two calls
 * on the same graph must not overlap on different streams. */
gsr_status_t gsr_spmm(const gsr_graph_t* g, const float* x, int64_t ldx, int32_t width, float* y,
                      int64_t ldy, int32_t transpose, void* stream);

/* gsr_spmm for callers that cannot allocate device memory or let a library do it on their behalf: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical
 * results; the scratch gsr_spmm keeps in the graph (the tile counters of its sweep and the first-pass sums of split
 * rows) lives in a fixed device array of the library instead, 4.1 MiB per GPU, held until the process ends.  The call
 * allocates and frees nothing and only launches kernels.  Limits: at most 16,384 first-pass chunks (rows above
 * "hub_threshold" stored entries, cut every "hub_chunk"), else GSR_ERR_UNSUPPORTED; the graph's device must be the
 * current one.  All calls on one GPU share the array: two that overlap (different streams or threads) race. */
gsr_status_t gsr_spmm_noalloc(const gsr_graph_t* g, const float* x, int64_t ldx, int32_t width, float* y,
                              int64_t ldy, int32_t transpose, void* stream);

/* H = A * scatter(V, I): the forward block's aggregation of a compressed embedding, Section
 * 4.1 eq. (10), every neighbour contributing at its own recorded columns.  vals: device n*k
 * of `dtype`; idx: device n*k int32 (distinct per row, any order); dg in {32, 64};
 * h_out: device n*dg float32 (dense).  workspace: device scratch of at least
 * gsr_spmm_compressed_workspace() bytes.  Synchronises the stream once to report indices
 * that are out of range or repeated (GSR_ERR_INVALID_ARG) instead of reading out of bounds. */
size_t gsr_spmm_compressed_workspace(const gsr_graph_t* g, int32_t k, int32_t dg);
gsr_status_t gsr_spmm_compressed(const gsr_graph_t* g, const void* vals, const int32_t* idx, int32_t k,
                                 int32_t dg, int32_t dtype, float* h_out, void* workspace,
                                 size_t workspace_bytes, void* stream);

/* ---- layers and the step ----
 *
 * Bytes of device workspace the layer / step calls need for (cfg, g).  gsr_step's figure
 * includes its activation and gradient arena and does not grow with cfg->l (the reversible
 * scheme's memory is independent of depth, Sections 1 and 2) unless cfg->save_indices is set. */
gsr_status_t gsr_workspace_size(const gsr_config_t* cfg, const gsr_graph_t* g, size_t* layer_bytes,
                                size_t* step_bytes);

/* eq. (6), in place: x_inout (device, N x D of cfg->dtype in cfg->layout) holds X on entry and
 * Y = Concat(Y_1..Y_C) on return.  w: device, C matrices dg x dg float32. */
gsr_status_t gsr_layer_forward(const gsr_graph_t* g, const gsr_config_t* cfg, const float* w,
                               void* x_inout, void* workspace, size_t workspace_bytes, void* stream);

/* eq. (7), in place: y_inout holds Y on entry and X on return (groups C..2, then Y_0, then 1). */
gsr_status_t gsr_layer_inverse(const gsr_graph_t* g, const gsr_config_t* cfg, const float* w,
                               void* y_inout, void* workspace, size_t workspace_bytes, void* stream);

/* Backward of one layer fused with its inverse (Algorithm 2's structure; eq. (3), eq. (11)):
 * y_inout: Y on entry, the rebuilt X on return; dy_inout: dL/dY on entry, dL/dX on return;
 * dw_out: device, C x dg x dg float32, overwritten with dL/dW_i.  Each block's input is
 * rebuilt and consumed once; gradients are read only at the positions recorded by I.
 * Needs a graph whose transpose is available (symmetric, or built by gsr_graph_create). */
gsr_status_t gsr_layer_backward(const gsr_graph_t* g, const gsr_config_t* cfg, const float* w,
                                void* y_inout, void* dy_inout, float* dw_out, void* workspace,
                                size_t workspace_bytes, void* stream);

/* One training step over cfg->l layers (Algorithm 1 then Algorithm 2; no parameter update):
 * forward sweep, scalar linear head + mean-squared-error loss, backward sweep with inverse
 * recomputation.  Nothing is kept per layer, except the column masks when cfg->save_indices is set.
 *   x0        device N x D (cfg->dtype, cfg->layout), read only
 *   w_all     device L x C x dg x dg float32
 *   w_out     device D float32;  b_out: device 1 float32;  target: device N float32
 *   loss_out  device 1 float32                      (required)
 *   yhat_out  device N float32                      (optional, may be NULL)
 *   dw_all    device L x C x dg x dg float32        (required)
 *   dw_out    device D float32;  db_out: device 1   (required)
 *   dx0_out, x0_rebuilt_out, xl_out: device N x D (cfg->dtype, cfg->layout), optional:
 *             dL/dX^0, the input as rebuilt by the inverse sweep, and X^L. */
gsr_status_t gsr_step(const gsr_graph_t* g, const gsr_config_t* cfg, const void* x0, const float* w_all,
                      const float* w_out, const float* b_out, const float* target, float* loss_out,
                      float* yhat_out, float* dw_all, float* dw_out, float* db_out, void* dx0_out,
                      void* x0_rebuilt_out, void* xl_out, void* workspace, size_t workspace_bytes,
                      void* stream);

/* Counts of the last gsr_step with cfg->save_indices == 2 that ran in `workspace` (same cfg and g): rows kept over
 * all blocks and layers, the largest number any one block listed, and the rows that were not kept because a block
 * listed more than cfg->tie_capacity.  Waits for `stream`.  Any output pointer may be NULL. */
gsr_status_t gsr_step_tie_stats(const gsr_graph_t* g, const gsr_config_t* cfg, const void* workspace,
                                int64_t* listed, int64_t* max_per_block, int64_t* dropped, void* stream);

/* The rows kept by that step for the input of block `block` (1..C) of layer `layer` (0..L-1), in no particular order:
 * rows_out (host, cfg->tie_capacity or its default entries) and masks_out (host, same count, bit c set: column c
 * kept); *count_out = entries written.  Waits for `stream`. */
gsr_status_t gsr_step_tie_export(const gsr_graph_t* g, const gsr_config_t* cfg, const void* workspace, int32_t layer,
                                 int32_t block, int32_t* rows_out, uint64_t* masks_out, int64_t* count_out, void* stream);

/* ---- the two-group pipeline as the walk-throughs of Sections 4.3 and 4.4 print it ----
 *
 * Its block differs from eq. (10): a row's slot-wise sums over its neighbours stand in the row's
 * OWN recorded columns, block(V, I)[i, I[i,t]] = sum_j a_ij V[j,t] (the printed block results of
 * Sections 4.3 and 4.4), and Algorithm 1 / 2 use it without weights.  float32 only; planes are
 * device n x dg with row stride ld elements, dg in [1, 64], 1 <= k <= dg.  workspace: device,
 * 256-byte aligned, at least gsr_walkthrough_workspace(g, k) bytes.  The products run through
 * gsr_spmm, so its note on overlapping calls applies.
 *
 * gsr_slot_block: out = block(vals, idx) (transpose = 1: sums over A^T).  vals: device n x k
 * float32, idx: device n x k int32; a column outside [0, dg) places nothing. */
size_t gsr_walkthrough_workspace(const gsr_graph_t* g, int32_t k);
gsr_status_t gsr_slot_block(const gsr_graph_t* g, const float* vals, const int32_t* idx, int32_t k, int32_t dg,
                            int32_t transpose, float* out, int64_t ld, void* workspace, size_t workspace_bytes,
                            void* stream);

/* One pass of the loop body of Algorithm 1, in place: x1 is the group that enters the first
 * GS-Op.  (V1, I1) = GS(x1); x2 += block(V1, I1); (V2, I2) = GS(x2); x1 = scatter(V1, I1) +
 * block(V2, I2). */
gsr_status_t gsr_alg1_layer_forward(const gsr_graph_t* g, int32_t dg, int32_t k, float* x1_inout, float* x2_inout,
                                    int64_t ld, void* workspace, size_t workspace_bytes, void* stream);

/* One pass of the loop body of Algorithm 2, in place, step by step as printed: (V2, I2) = GS(g2);
 * M1 = g1 - block(V2, I2); (V1, I1) = GS(M1); M2 = scatter(V2, I2) - block(V1, I1);
 * g1 = backward_block(M1, I1), g2 = backward_block(M2, I2), where backward_block(M, I) reads M
 * only at the recorded positions, sums over A^T and places at the row's recorded positions
 * (Section 4.1, eq. (11)). */
gsr_status_t gsr_alg2_layer_backward(const gsr_graph_t* g, int32_t dg, int32_t k, float* g1_inout, float* g2_inout,
                                     int64_t ld, void* workspace, size_t workspace_bytes, void* stream);

/* ---- parameter updates (Section 5 trains for 250 epochs; the optimiser is not named) ----
 *
 * Element-wise, in place, float32 device arrays of `count` elements; apply them to w_all, w_out and
 * b_out with the gradients gsr_step returned to make a full training step.
 * gsr_sgd_update:   w <- w - lr * (dw + weight_decay * w)
 * gsr_adam_update:  g = dw + weight_decay * w;  m <- beta1 m + (1 - beta1) g;  v <- beta2 v + (1 - beta2) g^2;
 *                   w <- w - lr * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps)   (Kingma & Ba, Algorithm 1);
 *                   m, v: device state of `count` floats, zero before step t = 1; t counts from 1. */
gsr_status_t gsr_sgd_update(float* w, const float* dw, int64_t count, float lr, float weight_decay, void* stream);
gsr_status_t gsr_adam_update(float* w, const float* dw, float* m, float* v, int64_t count, int64_t t, float lr,
                             float beta1, float beta2, float eps, float weight_decay, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GSR_H_ */
