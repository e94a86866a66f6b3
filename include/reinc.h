/*
 * reinc.h -- C ABI of libreinc_hip.so: the single-GPU hot path of incremental dynamic-GNN training
 * (ReInc, arXiv 2501.15348) written for AMD MI355X (gfx950).
 *
 * The method (paper Section 3.2): a dynamic graph is a series of snapshots G_t with node features
 * F_t over a fixed node set.  Instead of aggregating every snapshot from scratch (Eq. 1,
 * Agg_t = F_t *aggr G_t) the aggregate of snapshot t is derived from the cached aggregate of
 * snapshot t-1 and two small delta graphs (Eq. 2, Agg_t = Agg_{t-1} - F_{t-1} *aggr G-_t + F_t *aggr G+_t).
 * The aggregate feeds a GCN update (linear map + ReLU, Section 3.5 Listing 1) and, per node, a GRU
 * or LSTM over the snapshots of a sliding window (Section 2.2).
 *
 * Conventions
 *   - An edge (u -> v) goes from source u to target v and the TARGET aggregates the source's row.
 *     Adjacency is stored as CSR by destination: row v lists the sources of v's in-edges, ascending.
 *   - A snapshot is a SET of edges with u != v.  self_loop = 1 adds the identity to every snapshot.
 *   - deg_t(v) = self_loop + in-degree of v in snapshot t.
 *     Y_t = P_t X_t,  S_t = (A_t + self_loop I) Y_t,  Agg_t = Q_t S_t  with
 *       SUM : P = Q = I        MEAN: P = I, Q = 1/deg        SYM : P = Q = deg^(-1/2)      (deg = 0 -> 0)
 *   - All matrices are dense row-major.  Node ids are int32, 0 <= id < num_nodes <= 2^30.
 *     Row pointers are int64.  Feature storage is fp32 or bf16 (raw 16-bit patterns); every
 *     accumulator, aggregate, activation, weight and gradient is fp32.
 *   - "device" pointers are HIP device memory of the context's GPU; "host" pointers are ordinary
 *     host memory.  The caller owns every pointer it passes.  The library owns only what it carves
 *     out of the caller-provided arena and its host-side bookkeeping (released by reinc_destroy).
 *     No entry point calls hipMalloc or hipFree.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls marked ASYNC only
 *     enqueue work on it; calls marked SYNC return after the device work has finished.
 *   - Every function returns REINC_OK or a negative code and never throws or aborts;
 *     reinc_last_error() gives the text of the last failure on that context.
 *
 * Flat parameter / gradient vector used by the window calls (fp32, device):
 *   for l = 1..num_gcn_layers:  W_l [dims[l-1], dims[l]],  b_l [dims[l]]
 *   then the recurrent cell:    W_i [dims[last], K*H],  W_h [H, K*H],  b_i [K*H],  b_h [K*H]
 *   with K = 3 (GRU, gate order r,z,n) or 4 (LSTM, gate order i,f,g,o) and H = rnn_hidden.
 */
#ifndef REINC_H
#define REINC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define REINC_OK 0
#define REINC_E_ARG (-1)         /* bad argument (null pointer, id out of range, bad size) */
#define REINC_E_STATE (-2)       /* call out of order (snapshot not loaded, deltas not built, ...) */
#define REINC_E_NOMEM (-3)       /* the arena is too small */
#define REINC_E_HIP (-4)         /* a HIP call failed */
#define REINC_E_UNSUPPORTED (-5) /* valid request that this build does not implement */

#define REINC_AGG_SUM 0
#define REINC_AGG_MEAN 1
#define REINC_AGG_SYM 2

#define REINC_RNN_GRU 0
#define REINC_RNN_LSTM 1

#define REINC_F32 0
#define REINC_BF16 1

#define REINC_MAX_GCN_LAYERS 3

typedef struct reinc_ctx reinc_ctx; /* opaque */

typedef struct reinc_config {
    uint32_t struct_size;   /* sizeof(reinc_config): versions the struct */
    int32_t device;         /* HIP device ordinal */
    int64_t num_nodes;      /* N, fixed over the sequence (isolated nodes pad a varying node set, Section 3.2) */
    int32_t num_snapshots;  /* T */
    int32_t num_gcn_layers; /* 1..REINC_MAX_GCN_LAYERS */
    int32_t dims[REINC_MAX_GCN_LAYERS + 1]; /* dims[0] = feature width, dims[l] = width after layer l */
    int32_t rnn_kind;       /* REINC_RNN_* */
    int32_t rnn_hidden;     /* H */
    int32_t agg_kind;       /* REINC_AGG_* */
    int32_t self_loop;      /* 0 or 1 */
    int32_t feat_dtype;     /* REINC_F32 or REINC_BF16: storage type of the node features */
    float fallback_ratio;   /* window driver: use the from-scratch path for step t when
                               effective_delta_edges(t) / |E_t| exceeds this (Section 3.2, "user-defined
                               threshold").  < 0: never fall back.  0: always from scratch. */
    void *arena;            /* device memory owned by the caller, 256-byte aligned */
    uint64_t arena_bytes;
} reinc_config;

/* Sizes of the delta structures of one step t-1 -> t (all counts of entries). */
typedef struct reinc_delta_info {
    int64_t num_edges_prev, num_edges_cur; /* |E_{t-1}|, |E_t| */
    int64_t n_ins, n_del;                  /* |E_t \ E_{t-1}|, |E_{t-1} \ E_t| */
    int64_t n_changed;                     /* |C_t|: nodes whose scaled feature row Y changed */
    int64_t n_fchg_entries;                /* entries of (A_t + self_loop I) restricted to columns in C_t */
    int64_t n_rows;                        /* |R_t|: rows of S that can differ from step t-1 */
    int64_t n_entries;                     /* n_ins + n_del + n_fchg_entries: effective delta edges */
} reinc_delta_info;

typedef struct reinc_stats {
    int64_t arena_used, arena_peak;      /* bytes */
    int64_t global_hits, global_misses;  /* layer-1 aggregate cache (window driver) */
    int64_t steps_incremental, steps_full, steps_fallback;
    int64_t delta_entries_processed;     /* effective delta edges consumed by incremental steps */
    int64_t local_bytes;                 /* bytes of per-window activations currently held */
    /* budgeted layer-1 cache (reinc_cache_configure; all zero while every aggregate is kept) */
    int64_t global_admitted, global_refused, global_evicted, global_expired;
    int64_t global_bytes, global_peak_bytes; /* bytes the retained aggregates take now / at most so far */
} reinc_stats;

const char *reinc_version(void);

/* Creates a context on cfg->device.  Nothing is allocated on the device: all device storage is carved
 * out of cfg->arena.  SYNC. */
int reinc_create(reinc_ctx **out, const reinc_config *cfg);
int reinc_destroy(reinc_ctx *ctx);
/* Text of the most recent failure on ctx (valid until the next call on ctx); "" if none. */
const char *reinc_last_error(const reinc_ctx *ctx);
/* Arena bytes still free. */
int reinc_arena_free_bytes(const reinc_ctx *ctx, uint64_t *out);

/* ---- load the snapshot sequence (Section 2.1: snapshots G_t with features F_t) --------------------------
 * reinc_load_edges: src/dst are arrays of nnz int32 endpoints in any order, in HOST memory (on_device = 0) or in
 * DEVICE memory (on_device = 1).  Duplicates and self-loops are removed; ids outside [0, N) give REINC_E_ARG.  The
 * list is copied into the arena, where the canonical CSR (by destination) and CSC (by source) of snapshot t are
 * built (key sort, de-duplication); the caller's arrays are not kept.  SYNC.  Each snapshot is loaded once. */
int reinc_load_edges(reinc_ctx *ctx, int32_t t, const int32_t *src, const int32_t *dst, int64_t nnz, int on_device);
/* X_t = the given [N, dims[0]] matrix (fp32, or bf16 bit patterns when feat_dtype is bf16).
 * on_device selects whether X is a device or a host pointer.  SYNC. */
int reinc_load_features_full(reinc_ctx *ctx, int32_t t, const void *X, int on_device);
/* X_t = X_{t-1} with `rows` (HOST, sorted, unique, nrows entries) replaced by the rows of `vals`
 * (HOST, [nrows, dims[0]]).  Only the changed rows cross the host-device link (Section 4, delta mode).
 * Needs X_{t-1}.  SYNC. */
int reinc_load_features_delta(reinc_ctx *ctx, int32_t t, const int32_t *rows, int64_t nrows, const void *vals);

/* ---- per-snapshot deltas (Section 3.2: delta graphs G-_t, G+_t) ------------------------------------------
 * Builds, on the device, for step t (1 <= t < T; t < 0 = every step whose inputs are loaded):
 *   - the insert CSR  E_t \ E_{t-1} and the delete CSR E_{t-1} \ E_t (by destination, ascending columns);
 *   - the change set C_t = { u : X_t[u] != X_{t-1}[u] bitwise } (plus, for SYM, every u whose degree changed),
 *     ascending, and dY = P_t X_t - P_{t-1} X_{t-1} on those rows;
 *   - the merged signed delta rows used by reinc_aggregate_incremental: for each row v, first the inserted
 *     sources, then the deleted sources, then the sources u in C_t of v's in-edges at t (and v itself when
 *     self_loop is set and v is in C_t, placed last), each group ascending;
 *   - R_t, the ascending list of rows with at least one entry.
 * Needs edges and features of snapshots t-1 and t.  SYNC (sizes are read back to carve the arena). */
int reinc_build_deltas(reinc_ctx *ctx, int32_t t, void *stream);
int reinc_get_delta_info(reinc_ctx *ctx, int32_t t, reinc_delta_info *out);
/* Copies the insert (kind 0) or delete (kind 1) CSR of step t to HOST buffers: row_ptr[N+1], col[nnz].
 * Either buffer may be NULL; *nnz_out (may be NULL) receives the entry count, so a first call with NULL
 * buffers sizes the second.  SYNC. */
int reinc_get_delta_csr(reinc_ctx *ctx, int32_t t, int kind, int64_t *row_ptr, int32_t *col, int64_t *nnz_out);
/* Copies the merged structures of step t to HOST buffers (each may be NULL): entry_ptr[N+1];
 * entries[n_entries], each (kind << 30) | payload with kind 0 = inserted source id, 1 = deleted source id,
 * 2 = position in `changed` of a changed source; rows[n_rows]; changed[n_changed].  SYNC. */
int reinc_get_merged_delta(reinc_ctx *ctx, int32_t t, int64_t *entry_ptr, uint32_t *entries, int32_t *rows,
                           int32_t *changed);
/* Copies snapshot t's canonical CSR (transpose = 0) or CSC (transpose = 1) to HOST buffers.  SYNC. */
int reinc_get_snapshot_csr(reinc_ctx *ctx, int32_t t, int transpose, int64_t *ptr, int32_t *idx, int64_t *nnz_out);

/* ---- aggregation ------------------------------------------------------------------------------------------
 * reinc_aggregate_full (Section 3.2, Eq. 1), ASYNC.  X: device [N, d] of x_dtype, or NULL for the stored X_t
 * (then d and x_dtype must match the stored features).  out: device fp32 [N, d].
 *   transpose = 0:  out = S_t = (A_t + sI) P_t X          (apply_q = 0)
 *                   out = Agg_t = Q_t S_t                 (apply_q = 1)
 *   transpose = 1:  out = P_t (A_t + sI)^T (Q_t X)  if apply_q, else P_t (A_t + sI)^T X: the adjoint used
 *                   by the backward pass (X is then the gradient w.r.t. Agg or S).
 * d * sizeof(element) must be a power of two between 16 and 1024 bytes. */
int reinc_aggregate_full(reinc_ctx *ctx, int32_t t, int transpose, const void *X, int x_dtype, int32_t d,
                         int apply_q, float *out, void *stream);
/* reinc_aggregate_incremental (Section 3.2, Eq. 2), ASYNC.  Derives S_t of the stored features from
 * S_{t-1}:  for every row r in R_t
 *     S_t[r] = S_{t-1}[r] + sum_{inserted u} Y_{t-1}[u] - sum_{deleted u} Y_{t-1}[u] + sum_{changed u} dY[u]
 * and S_t[r] = S_{t-1}[r] elsewhere.  S_prev, S_out: device fp32 [N, dims[0]].  S_out may be S_prev itself
 * (in place: only rows in R_t are touched) or a disjoint buffer (all rows are written).  Needs
 * reinc_build_deltas(t).  agg_out (may be NULL; in-place calls only): device fp32 [N, dims[0]]; its rows in R_t
 * receive Q_t S_t and its other rows are left alone, so a buffer that held Agg_{t-1} holds Agg_t afterwards (a
 * row outside R_t keeps both its sum and its degree). */
int reinc_aggregate_incremental(reinc_ctx *ctx, int32_t t, const float *S_prev, float *S_out, float *agg_out,
                                void *stream);

/* ---- max / min aggregation (Section 3.2: aggregators that cannot be updated by subtraction) ----------------
 * For target v and feature j, over the sources u of v's in-edges at snapshot t (and v itself when self_loop is
 * set):  M[v, j] = max_u X[u, j] (REINC_OP_MAX) or min_u X[u, j] (REINC_OP_MIN), and C[v, j] = the source that
 * attains it -- it names the contributing edge (C[v, j] -> v); among equal values the smallest id.  A target
 * without any source gets M = 0 and C = -1.  No degree scaling is applied.
 *
 * reinc_aggregate_full_minmax, ASYNC: from scratch.  X, x_dtype, d as for reinc_aggregate_full (NULL = the stored
 * features); out: device fp32 [N, d]; contrib: device int32 [N, d].
 *
 * reinc_aggregate_incremental_minmax, ASYNC: (M_t, C_t) of the stored features from (M_{t-1}, C_{t-1}), the
 * paper's procedure: for every row of R_t, if a deleted edge or a changed source is the recorded contributor of
 * any feature of the row, the row is aggregated from scratch; otherwise the previous result is combined with the
 * values that arrive over inserted edges and from changed sources.  (A contributor that an arriving value has
 * already replaced does not count as lost; rows with more than 64 delta entries are aggregated from scratch
 * without looking.)  The outputs may be the previous buffers themselves (in place: only rows of
 * R_t are touched) or disjoint buffers (every row is written); values and contributors must agree on that.
 * work: device int32 [2 N + 4] scratch; on completion work[0] = number of rows aggregated from scratch.
 * Needs reinc_build_deltas(t); the context's agg_kind only matters in that SYM adds the degree-changed nodes to
 * the change set (more rows are then re-examined; results are the same). */
#define REINC_OP_MAX 0
#define REINC_OP_MIN 1
int reinc_aggregate_full_minmax(reinc_ctx *ctx, int32_t t, int op, const void *X, int x_dtype, int32_t d, float *out,
                                int32_t *contrib, void *stream);
int reinc_aggregate_incremental_minmax(reinc_ctx *ctx, int32_t t, int op, const float *M_prev, const int32_t *C_prev,
                                       float *M_out, int32_t *C_out, int32_t *work, void *stream);
/* reinc_aggregate_incremental_minmax_static, ASYNC: the same step for callers that cannot allocate device memory
 * or provide a work buffer (code under HIP graph capture, tight serving loops, harnesses that forbid allocation).
 * The work area is a static device array inside the library (8 MiB per GPU, held until the process ends); the call
 * allocates nothing and enqueues kernels only.  At most 2^20 nodes: a larger context gets REINC_E_ARG (use the
 * call above).  n_redone_out: device int32 scalar that receives the number of rows aggregated from scratch, or NULL.
 * All calls on one GPU share the one work area: calls that may overlap on a GPU (different streams, different
 * contexts or threads) race and must be serialised by the caller.  Other arguments, results and errors as above. */
int reinc_aggregate_incremental_minmax_static(reinc_ctx *ctx, int32_t t, int op, const float *M_prev,
                                              const int32_t *C_prev, float *M_out, int32_t *C_out,
                                              int32_t *n_redone_out, void *stream);

/* ---- dense steps ------------------------------------------------------------------------------------------
 * reinc_gcn_transform (Section 3.5, Listing 1: update = ReLU(linear(aggregate))), ASYNC.
 *   out[n, d_out] = act( (row_scale .* A)[n, d_in] * W[d_in, d_out] + b )
 * A: device fp32 (a_dtype REINC_F32) or bf16; row_scale: device fp32 [n] or NULL; b: device [d_out] or NULL;
 * relu: 0/1; out: device fp32. */
int reinc_gcn_transform(reinc_ctx *ctx, const void *A, int a_dtype, int64_t n, int32_t d_in, int32_t d_out,
                        const float *row_scale, const float *W, const float *b, int relu, float *out, void *stream);
/* reinc_rnn_step: one GRU (3 gates) or LSTM (4 gates) step for n independent nodes (Section 2.1: the RNN
 * runs per node over time; gate counts: Section 3.3), ASYNC.
 *   GRU : r = sig(x W_ir + b_ir + h W_hr + b_hr), z likewise, n = tanh(x W_in + b_in + r .* (h W_hn + b_hn)),
 *         h' = (1 - z) .* n + z .* h
 *   LSTM: (i, f, g, o) = (sig, sig, tanh, sig)(x W_i + b_i + h W_h + b_h),  c' = f .* c + i .* g,  h' = o .* tanh(c')
 * x [n, d_in], h_prev/h_out [n, H], c_prev/c_out [n, H] (LSTM only, else NULL), W_i [d_in, K*H], W_h [H, K*H],
 * b_i, b_h [K*H]; all device fp32.  h_prev (and c_prev) may be NULL for a zero state.  h_out may not alias h_prev.
 * saved (may be NULL): device fp32 [n, 4*H] (GRU: r, z, n, h W_hn + b_hn) or [n, 4*H] (LSTM: i, f, g, o),
 * kept for the backward pass. */
int reinc_rnn_step(reinc_ctx *ctx, int rnn_kind, const float *x, int64_t n, int32_t d_in, int32_t H,
                   const float *h_prev, const float *c_prev, const float *W_i, const float *W_h, const float *b_i,
                   const float *b_h, float *h_out, float *c_out, float *saved, void *stream);

/* ---- window driver (Section 2.2: a window of L consecutive snapshots is one sample; Section 3.3: caches) -----
 * reinc_forward_window, ASYNC: runs snapshots t0 .. t0+L-1 through the GCN layers and the recurrent cell
 * from a zero state.  The layer-1 sums S_t of the stored features are weight-independent; they are kept in
 * the global cache for every t once computed (by Eq. 2 from S_{t-1} when that is cached and the step is under
 * fallback_ratio, else by Eq. 1) and reused by every later window.  Per-window activations go to the local
 * cache and stay there until the next forward call.  target: device [N, H] or NULL;
 * loss_out: device scalar = mean((h_last - target)^2) (ignored if target is NULL); h_last: device [N, H] or NULL. */
int reinc_forward_window(reinc_ctx *ctx, int32_t t0, int32_t L, const float *params, const float *target,
                         float *loss_out, float *h_last, void *stream);
/* reinc_backward_window, ASYNC: back-propagation through time for the window of the preceding
 * reinc_forward_window call (same t0, L, params, target).  grads: device, same layout as params, overwritten. */
int reinc_backward_window(reinc_ctx *ctx, int32_t t0, int32_t L, const float *params, const float *target,
                          float *grads, void *stream);
/* The integrated model (Section 2.1: a GraphRNN replaces the matrix products inside the recurrent gates by graph
 * operations on x_t and h_{t-1}; Section 3.1, reuse across gates: both are aggregated once per timestep and all
 * gates share the two aggregates).  Per timestep
 *     ax = Agg(X_t; G_t)      -- the layer-1 aggregate of the stored features: global cache / Eq. 2, as above
 *     ah = Agg(h_{t-1}; G_t)  -- from scratch (the state changes everywhere), kept in the local cache
 *     gates from ax W_i + b_i and ah W_h + b_h with the cell equations of reinc_rnn_step, the carry term on the
 *     un-aggregated state:  GRU h_t = (1 - z) n + z h_{t-1};  LSTM c_t = f c_{t-1} + i g, h_t = o tanh(c_t).
 * The GCN layer fields of the configuration are not used (dims[0] is the feature width).  params / grads: W_i
 * [dims[0], K*H], W_h [H, K*H], b_i [K*H], b_h [K*H], flat in this order.  rnn_hidden * 4 must be a power of two
 * between 16 and 1024 bytes.  Other arguments and the ASYNC / state rules as for reinc_forward_window /
 * reinc_backward_window (the backward call needs the integrated forward call of the same window). */
int reinc_forward_window_integrated(reinc_ctx *ctx, int32_t t0, int32_t L, const float *params, const float *target,
                                    float *loss_out, float *h_last, void *stream);
int reinc_backward_window_integrated(reinc_ctx *ctx, int32_t t0, int32_t L, const float *params, const float *target,
                                     float *grads, void *stream);
/* params[i] -= lr * grads[i] for count fp32 values (plain SGD; the paper names no optimiser), ASYNC. */
int reinc_sgd_step(reinc_ctx *ctx, float *params, const float *grads, int64_t count, float lr, void *stream);
/* Drops every cached layer-1 sum (the next windows recompute them). */
int reinc_cache_clear(reinc_ctx *ctx);
/* Drops everything derived from the loaded snapshots -- deltas, cached sums, the local cache -- and returns
 * their arena space, so that the next reinc_build_deltas / window calls start cold.  Fails with REINC_E_STATE
 * if a snapshot was loaded after the first derived structure was built.  SYNC. */
int reinc_reset_derived(reinc_ctx *ctx);
/* Device pointer of the cached layer-1 sums S_t ([N, dims[0]] fp32; in a context filled by reinc_batch_load only the
 * first rows, see there) or NULL if not cached.  With a cache budget the pointer is good until the next forward-window
 * call (an aggregate the policy does not keep lives that long). */
int reinc_cache_peek(reinc_ctx *ctx, int32_t t, const float **S_out);

/* ---- node mini-batches (Section 4.2, "Rethinking Mini-batch Training") -------------------------------------
 * A sample is the sequence of computational graphs of a set of selected nodes.  With F_0 = the batch and
 * F_k = F_{k-1} plus the sources of every edge, of any snapshot, whose target is in F_{k-1}, the sub-sequence of a
 * batch keeps the nodes F_hops and, of every snapshot, the edges whose target is in F_{hops-1}; its nodes are
 * numbered batch first (in the order given), then the nodes first reached in one hop by ascending id, then those
 * first reached in two hops, and so on: every F_k is the first |F_k| ids.  A stacked model of `hops`
 * aggregation layers evaluated on the sub-sequence gives on the batch rows exactly what it gives on the whole
 * graph.  (The degree scales of the mean and symmetric normalisations are carried over from the source graph, so
 * the degree of a node whose own in-edges are not kept -- a source only -- is still the right one.)  The integrated
 * model (Section 2.1) aggregates the hidden state inside the gates, so a batch row depends on one hop more per
 * timestep: a window of L timesteps is exact on a sub-sequence planned with hops >= L.  On a batch context its window
 * calls compute timestep i of L on the nodes within L - 1 - i hops of the batch (the last one on the batch rows),
 * reinc_forward_window_integrated writes rows [0, n_batch) of h_last only, and the cached input sums hold the rows of
 * the first timestep (sums cached with fewer rows, by the stacked model or a shorter window, are recomputed).
 *
 * The sub-sequence goes into a second context, which is then used like any other: sliding its windows over the
 * whole sequence before the next batch is extracted (seq-first) lets its aggregate cache serve every window and
 * hold the rows of this batch only.
 *
 * reinc_batch_plan: nodes = HOST array of n_batch distinct ids; hops <= 0 selects num_gcn_layers.  Every
 *   snapshot's edges must be loaded.  Computes the node set on the device and keeps it in
 *   `ctx` (3 ints per node of arena space, allocated by the first plan) until the next plan; returns the number of
 *   nodes of the sub-sequence and |F_{hops-1}|.  REINC_E_ARG for ids out of range or listed twice.  SYNC.
 * reinc_batch_node_list: old id of every node of the planned sub-sequence, to a HOST array of n_nodes int32.  SYNC.
 * reinc_batch_load: fills `child` -- created by the caller with num_nodes = the planned count, the same
 *   num_snapshots, dims[0], feat_dtype, agg_kind, self_loop and device, no snapshots loaded -- with the extracted
 *   edges, the gathered feature rows and degree scales of every snapshot, and sets its loss rows to n_batch.  It
 *   also tells `child` on how many of its first rows each layer below the last is needed (layer l of L: |F_{L-l}|):
 *   the window calls compute a layer on those rows only, and the cached layer-1 sums of `child` hold the rows that
 *   layer 1 is needed on only (reinc_cache_peek then returns that many rows).  Environment variable
 *   REINC_LAYER_ROWS = megabytes a restriction must leave out per timestep to be taken (default 0).  Errors are
 *   reported on `ctx`; after a failure `child` may hold some of the snapshots and is good for reinc_destroy only.
 *   Both contexts stay independent afterwards (the child holds copies).  SYNC.
 * reinc_set_loss_rows: the loss of the window calls becomes the mean over rows [0, rows) of h_last and target
 *   (both stay [N, H]); the gradients are those of that loss.  The stacked model then computes its last GCN layer
 *   and the recurrent cell on those rows only (nothing else depends on the others), and reinc_forward_window writes
 *   rows [0, rows) of h_last only.  rows = 0 or N: every row (the default).  A backward call needs a forward call
 *   made with the same rows (REINC_E_STATE otherwise).  Forgets what reinc_batch_load said about the layers below and
 *   about the timesteps of the integrated model (and with it the cached sums of a batch context, which hold some
 *   rows only). */
int reinc_batch_plan(reinc_ctx *ctx, const int32_t *nodes, int64_t n_batch, int32_t hops, int64_t *n_nodes_out,
                     int64_t *n_inner_out);
int reinc_batch_node_list(reinc_ctx *ctx, int32_t *out);
int reinc_batch_load(reinc_ctx *ctx, reinc_ctx *child);
int reinc_set_loss_rows(reinc_ctx *ctx, int64_t rows);

/* ---- cache budget and eviction policy (Section 3.3, "Eviction Policy"; compared with LRU / LFU in Section 5) ----
 * By default every layer-1 aggregate stays cached (REINC_POLICY_KEEP_ALL: T * N * dims[0] * 4 bytes in the end).
 * reinc_cache_configure limits what is RETAINED BETWEEN WINDOWS to budget_bytes and chooses who leaves:
 *   REINC_POLICY_SCORE  the paper's rule: score = F / S - I, lowest score leaves first, and an aggregate that no
 *                       later window needs (F = 0) leaves at once.  For the aggregate of snapshot t computed by the
 *                       window that starts at t0, in an epoch of windows t0 = 0, stride, 2*stride, ... of length
 *                       `window` over the T snapshots:
 *                         F = min((t - t0) / stride, (T - window - t0) / stride)   later windows that contain t
 *                         I = window - stride                                     the paper's encoder imminence
 *                         S = N * dims[0] * 4 bytes
 *                       (the paper prints F for its encoder-decoder model and stride 1; this is the same count for a
 *                       model without a decoder).  A newcomer that scores no higher than what it would displace is
 *                       not kept.
 *   REINC_POLICY_LRU / REINC_POLICY_LFU   always keep the newcomer; the least recently / least frequently (since
 *                       it entered; ties: least recently) used aggregate leaves.
 * Mechanics: a window looks up its snapshots in order; what it has to compute lives in a buffer of its own until the
 * next forward-window call begins, and is offered to the policy then, in snapshot order (so the backward pass of the
 * window still finds it).  Device memory: (budget_bytes / S + window) buffers of S bytes, taken from the arena at
 * the first window; no copies are made.  Windows longer than `window` are refused while a budget is set.
 * The call drops every cached aggregate.  Results do not depend on the policy beyond rounding (an aggregate that
 * was not kept is recomputed, from scratch or from its predecessor); the counters in reinc_stats do. */
#define REINC_POLICY_KEEP_ALL 0
#define REINC_POLICY_SCORE 1
#define REINC_POLICY_LRU 2
#define REINC_POLICY_LFU 3
int reinc_cache_configure(reinc_ctx *ctx, int32_t policy, int64_t budget_bytes, int32_t window, int32_t stride);

/* The same policies as a stand-alone store of (key, size, F, I) records, HOST only, no device and no context needed:
 * a trace of look-ups and offers can be replayed to size a budget before training.
 *   access:  *hit = 1 and one future access consumed (recency / frequency refreshed; under REINC_POLICY_SCORE the
 *            entry leaves when its F reaches 0), or *hit = 0 and nothing changes.
 *   offer:   after a miss.  *admitted tells whether the record was kept; the keys that left for it are written to
 *            evicted[0 .. min(*n_evicted, evicted_cap)) (NULL / 0 to ignore).  A refused offer evicts nothing.  An
 *            offer of a present key only replaces its F and I.  size > 0.
 *   rescore: replaces F and I of a present key (under REINC_POLICY_SCORE, F <= 0 expires it).
 *   counters: out[REINC_POLICY_COUNTERS] = hits, misses, admitted, refused, evicted, expired, used, peak_used.
 * Ties: the older last use leaves first, then the smaller key.  Scores are compared exactly (no floating point);
 * sizes, F and I must stay below 2^40. */
typedef struct reinc_policy reinc_policy;
#define REINC_POLICY_COUNTERS 8
int reinc_policy_create(reinc_policy **out, int32_t policy, int64_t budget);
int reinc_policy_destroy(reinc_policy *p);
int reinc_policy_access(reinc_policy *p, int64_t key, int32_t *hit);
int reinc_policy_offer(reinc_policy *p, int64_t key, int64_t size, int64_t future, int64_t imminence, int32_t *admitted,
                       int64_t *evicted, int32_t evicted_cap, int32_t *n_evicted);
int reinc_policy_rescore(reinc_policy *p, int64_t key, int64_t future, int64_t imminence);
int reinc_policy_contains(const reinc_policy *p, int64_t key, int32_t *present);
int reinc_policy_counters(const reinc_policy *p, int64_t *out);
int reinc_get_stats(reinc_ctx *ctx, reinc_stats *out);

/* ---- kernel timing ------------------------------------------------------------------------------------------
 * Between reinc_profile_begin and reinc_profile_end every launch of a kernel class selected in `mask`
 * (bit REINC_K_*) is bracketed by a pair of HIP events on the stream it runs on.  reinc_profile_end waits for
 * the device (SYNC) and fills launches[k] and total_ms[k] for k < REINC_K_COUNT.  At most
 * REINC_PROFILE_MAX_LAUNCHES launches are recorded per session; later ones run untimed. */
#define REINC_K_AGG_FULL 0   /* wave-per-row gather of reinc_aggregate_full (forward and adjoint) */
#define REINC_K_AGG_INC 1    /* incremental row update */
#define REINC_K_GEMM_ROWS 2  /* row-tile GEMM (GCN update, input gradients) */
#define REINC_K_RNN 3        /* fused recurrent step */
#define REINC_K_REDUCE 4     /* weight-gradient reduction GEMM */
#define REINC_K_ELEM 5       /* elementwise recurrent backward */
#define REINC_K_DIFF 6       /* snapshot-diff count + fill */
#define REINC_K_AGG_MINMAX 7 /* max / min aggregation (from scratch or incremental: all kernels of a call) */
#define REINC_K_COUNT 8
#define REINC_PROFILE_MAX_LAUNCHES 16384
int reinc_profile_begin(reinc_ctx *ctx, uint32_t mask);
int reinc_profile_end(reinc_ctx *ctx, int64_t *launches, double *total_ms);

#ifdef __cplusplus
}
#endif
#endif /* REINC_H */
