// Internal state of libreinc_hip.so (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <memory>
#include <string>
#include <vector>

#include "reinc.h"
#include "cache_policy.h"

namespace reinc {

constexpr uint32_t kKindShift = 30;  // merged delta entry = (kind << 30) | payload
constexpr uint32_t kPayloadMask = (1u << kKindShift) - 1u;
constexpr int64_t kMaxNodes = int64_t(1) << kKindShift;
constexpr int kLongRow = 64;  // rows with more in-edges than this take the block-per-row path

// One canonical snapshot on the device.
struct Snapshot {
    bool edges_loaded = false;
    bool feats_loaded = false;
    bool feats_from_delta = false;
    int64_t nnz = 0;
    // CSR by destination and CSC by source
    int64_t *row_ptr = nullptr;
    int32_t *col = nullptr;
    int32_t *rowid = nullptr;  // target of every CSR entry (the expanded row pointer)
    int64_t *col_ptr = nullptr;
    int32_t *row = nullptr;
    // degree scalings: p (source side), q (target side), fp32 [N]
    float *p = nullptr;
    float *q = nullptr;
    // rows (columns) ordered by falling length: the order in which the group-per-row aggregation kernel takes them, so
    // that the rows a wavefront works on together are equally long (a wavefront lasts as long as its longest row)
    int32_t *row_order = nullptr, *col_order = nullptr;
    // rows / columns longer than kLongRow (ascending)
    int32_t *long_rows = nullptr;
    int32_t n_long_rows = 0;
    int32_t *long_cols = nullptr;
    int32_t n_long_cols = 0;
    // features [N, d0] in feat_dtype
    void *x = nullptr;
    // rows replaced by load_features_delta (device copy, ascending)
    int32_t *feat_rows = nullptr;
    int64_t n_feat_rows = 0;
};

// Delta structures of step t-1 -> t.
struct Delta {
    bool built = false;
    reinc_delta_info info{};
    int64_t *ins_ptr = nullptr;
    int32_t *ins_col = nullptr;
    int64_t *del_ptr = nullptr;
    int32_t *del_col = nullptr;
    int64_t *ent_ptr = nullptr;  // [N+1]
    uint32_t *ent = nullptr;     // [n_entries]
    int32_t *rows = nullptr;     // R_t [n_rows]
    int64_t *row_ent = nullptr;    // [n_rows + 1]: ent_ptr of the listed rows (their entries are adjacent)
    int32_t *changed = nullptr;  // C_t [n_changed]
    float *dY = nullptr;         // [n_changed, d0] fp32
};

// One aggregation problem: CSR-like (ptr, idx) over n rows, input rows X, optional source / target scalings and
// output mask, output rows, and the list of rows longer than kLongRow.
constexpr int kMaxAggBatch = 8;
struct AggItem {
    const int64_t *ptr;
    const int32_t *idx;
    const void *X;
    const float *in_scale, *out_scale, *mask;
    const float *add;  // [n, d] or null: added to the finished row (after scaling and masking)
    float *out;
    const int32_t *long_rows;
    int32_t n_long;
    int64_t row_limit = 0;  // > 0: listed long rows from this row on are skipped (their output rows do not exist)
    const int32_t *order = nullptr;  // [n] or null: the row the i-th lane group of the short-row kernel takes
    const float *bias = nullptr;     // [d] or null: added to the scaled row (before relu, mask and add)
    int relu = 0;                    // clamp at zero after the bias
};
struct AggBatch {
    int count = 0;
    AggItem item[kMaxAggBatch];
};

struct LocalStep {  // per-window activations of one timestep (local cache)
    float *S[REINC_MAX_GCN_LAYERS + 1] = {};  // S[l]: un-normalised sums feeding layer l (l >= 2; S[1] lives in the global cache)
    float *H[REINC_MAX_GCN_LAYERS + 1] = {};  // H[l]: output of layer l
    float *h = nullptr, *c = nullptr;         // recurrent state after this step
    float *saved = nullptr;                   // gate values [N, 4H]
};

}  // namespace reinc

struct reinc_ctx {
    reinc_config cfg{};
    std::string err;
    // arena: persistent allocations grow from the bottom, per-call scratch from the top
    char *base = nullptr;
    uint64_t size = 0, bottom = 0, top = 0, peak = 0;
    std::vector<reinc::Snapshot> snaps;
    std::vector<reinc::Delta> deltas;
    // global cache: where the layer-1 sums S^1_t of each snapshot are right now (null: nowhere)
    std::vector<float *> gcache;
    // budgeted global cache (reinc_cache_configure); gpolicy is null while every aggregate is kept
    std::unique_ptr<reinc::CachePolicy> gpolicy;
    int64_t budget_slots = 0;                 // buffers the policy may keep between windows
    int32_t plan_window = 0, plan_stride = 1; // the epoch the future access counts are derived from
    std::vector<float *> pool, pool_free;     // budget_slots + plan_window buffers of one aggregate each, and the free ones
    std::vector<int32_t> pending;             // snapshots the last window computed: offered when the next one begins
    std::vector<int32_t> expired_pending;     // hits of the last window that expired: their buffers return then too
    int32_t pending_t0 = 0, pending_L = 0;    // the window that computed `pending`
    void sync_policy_stats() {
        if (!gpolicy) return;
        const reinc::CachePolicy::Counters &k = gpolicy->counters();
        stats.global_admitted = k.admitted;
        stats.global_refused = k.refused;
        stats.global_evicted = k.evicted;
        stats.global_expired = k.expired;
        stats.global_bytes = k.used;
        stats.global_peak_bytes = k.peak_used;
    }
    // local cache
    std::vector<reinc::LocalStep> local;
    uint64_t local_reserved = 0;  // bytes at the top of the arena held by the local cache
    bool local_valid = false;
    int64_t local_top = -1;  // row count the top quantities of the local cache are placed for (see place_rows)
    int32_t local_t0 = -1, local_L = 0;  // start of the window the local cache holds; the longest window it is carved for
    int32_t local_len = 0;               // length of the window it holds (the last forward call's)
    int local_kind = 0;  // which model carved the local cache: 0 = stacked (GCN layers, then the cell), 1 = integrated
    float *zero_state = nullptr;  // [N, H] zeros: the recurrent state before the first timestep of a window
    float *q_block = nullptr;     // [T, N] target-side degree scales of all snapshots (null for SUM)
    int max_batch = reinc::kMaxAggBatch;  // timesteps the window driver handles per launch (REINC_BATCH=1..8 lowers it)
    float *loss_partial = nullptr;
    int64_t loss_rows = 0;  // rows [0, loss_rows) enter the loss (a node mini-batch, numbered first); 0 = every row
    int64_t counted_rows() const { return loss_rows > 0 ? loss_rows : cfg.num_nodes; }
    // The stacked model computes its last GCN layer and the recurrent cell on the loss rows only (nothing else reads
    // them).  The layers below need the batch's neighbourhood: layer l of L the nodes within L - l hops, which a batch
    // context numbers first (layer_rows[l] of them, set by reinc_batch_load; 0 = every row).
    int64_t top_rows() const { return counted_rows(); }
    int64_t layer_rows[REINC_MAX_GCN_LAYERS + 1] = {};
    int64_t rows_of_layer(int l) const
    {
        if (l == cfg.num_gcn_layers) return top_rows();
        return l >= 1 && layer_rows[l] > 0 ? layer_rows[l] : cfg.num_nodes;
    }
    // rows of the cached layer-1 sums that are computed and kept (a batch context: those layer 1 is needed on; the
    // buffers of the global cache are then that short); 0 = every row
    int64_t cache_rows = 0;
    int64_t cached_rows() const { return cache_rows > 0 ? cache_rows : cfg.num_nodes; }
    int64_t local_rows[REINC_MAX_GCN_LAYERS + 1] = {};  // rows_of_layer(l) the local cache is placed for (see place_rows)
    // A batch context: hop_rows[k] = nodes within k hops of the batch (its first ids), set by reinc_batch_load; empty =
    // unknown.  The integrated model, whose hidden state is aggregated once per timestep, needs timestep i of an
    // L-step window on the nodes within L - 1 - i hops only.
    std::vector<int64_t> hop_rows;
    int64_t integrated_rows(int32_t L, int32_t i) const
    {
        const int64_t k = int64_t(L) - 1 - i;
        if (loss_rows <= 0 || hop_rows.empty() || k >= int64_t(hop_rows.size())) return cfg.num_nodes;
        return hop_rows[size_t(k)];
    }
    std::vector<int64_t> step_rows;  // rows the last integrated forward pass computed per timestep (for its backward pass)
    // node mini-batch plan made on this context (reinc_batch_plan): hop level and new id per node, the node list
    int32_t *batch_level = nullptr, *batch_new_id = nullptr, *batch_nodes = nullptr;
    int64_t batch_size = 0, batch_total = 0;  // batch nodes, nodes of the sub-sequence (0: no plan)
    int32_t batch_hops = 0;
    std::vector<int64_t> batch_reach;  // [k] = nodes reached in at most k hops (the first ids of the sub-sequence)
    reinc_stats stats{};
    // arena bookkeeping for reinc_reset_derived
    bool has_derived = false, load_after_derived = false;
    uint64_t derived_mark = 0;
    void note_derived() {
        if (!has_derived) {
            has_derived = true;
            derived_mark = bottom;
        }
    }
    // kernel timing (reinc_profile_begin / _end)
    uint32_t prof_mask = 0;
    std::vector<hipEvent_t> prof_events;  // pool, two per recorded launch
    std::vector<int> prof_kind;           // kind of each recorded launch

    int fail(int code, const char *fmt, ...) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        err = buf;
        return code;
    }
    // persistent allocation (256-byte aligned); nullptr when the arena is exhausted
    void *alloc(uint64_t bytes) {
        uint64_t b = (bytes + 255) & ~uint64_t(255);
        if (bottom + b > top) return nullptr;
        void *p = base + bottom;
        bottom += b;
        if (bottom + (size - top) > peak) peak = bottom + (size - top);
        return p;
    }
    // scratch allocation, released by scratch_reset()
    void *scratch(uint64_t bytes) {
        uint64_t b = (bytes + 255) & ~uint64_t(255);
        if (bottom + b > top) return nullptr;
        top -= b;  // scratch sits below the local cache, which holds the last local_reserved bytes
        if (bottom + (size - top) > peak) peak = bottom + (size - top);
        return base + top;
    }
    void scratch_reset() { top = size - local_reserved; }
    int64_t N() const { return cfg.num_nodes; }
    int elem_bytes() const { return cfg.feat_dtype == REINC_BF16 ? 2 : 4; }
};

namespace reinc {
// Times launches of a kernel class when that class is being profiled.  Default: an event pair recorded around
// everything launched during the scope's lifetime.  With `attached`, nothing is recorded here; the caller hands
// start() / stop() to hipExtLaunchKernelGGL, which stamps them with the kernel's own begin and end.
struct ProfScope {
    reinc_ctx *ctx;
    hipStream_t s;
    int slot = -1;
    bool attached;
    ProfScope(reinc_ctx *c, int kind, hipStream_t st, bool attach = false) : ctx(c), s(st), attached(attach) {
        if (!(c->prof_mask & (1u << kind)) || c->prof_kind.size() >= REINC_PROFILE_MAX_LAUNCHES) return;
        const size_t need = 2 * (c->prof_kind.size() + 1);
        while (c->prof_events.size() < need) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) return;
            c->prof_events.push_back(e);
        }
        slot = int(c->prof_kind.size());
        c->prof_kind.push_back(kind);
        if (!attached) (void)hipEventRecord(c->prof_events[2 * slot], s);
    }
    ~ProfScope() {
        if (slot >= 0 && !attached) (void)hipEventRecord(ctx->prof_events[2 * slot + 1], s);
    }
    hipEvent_t start() const { return slot >= 0 ? ctx->prof_events[2 * slot] : nullptr; }
    hipEvent_t stop() const { return slot >= 0 ? ctx->prof_events[2 * slot + 1] : nullptr; }
    ProfScope(const ProfScope &) = delete;
    ProfScope &operator=(const ProfScope &) = delete;
};
}  // namespace reinc

#define REINC_HIP(ctx, expr)                                                                        \
    do {                                                                                            \
        hipError_t e_ = (expr);                                                                     \
        if (e_ != hipSuccess) return (ctx)->fail(REINC_E_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

#define REINC_TRY(expr)           \
    do {                          \
        int rc_ = (expr);         \
        if (rc_ != REINC_OK) return rc_; \
    } while (0)

namespace reinc {

// ---- api.hip
// reinc_load_edges with the raw list in host or in device memory
int load_edges(reinc_ctx *ctx, int32_t t, const int32_t *src, const int32_t *dst, int64_t nnz, bool on_device);
unsigned node_key_bits(int64_t n);  // bits that hold any id in [0, n]
// reinc_aggregate_incremental_minmax with the work area given by the caller of this function; `timed`: the launches
// may be bracketed by profiling events
int minmax_incremental(reinc_ctx *ctx, int32_t t, int op, const float *M_prev, const int32_t *C_prev, float *M_out,
                       int32_t *C_out, int32_t *work, bool timed, hipStream_t s);

// ---- noalloc.hip
// finds the address of the static work area on the context's device (once per device)
int static_scratch_init(reinc_ctx *ctx);

// ---- kernels_graph.hip
// exclusive scan of int32 counts [n] into int64 offsets [n+1]; tmp: scratch of scan_tmp_bytes(n)
uint64_t scan_tmp_bytes(int64_t n);
void launch_scan(const int32_t *counts, int64_t *offsets, int64_t n, void *tmp, hipStream_t s);
// Many exclusive scans in one launch.  Job j scans in[0, n) into out[0, n]; tile0 = scan_tiles() of all jobs before
// it.  jobs_dev: the job table in device memory; tile_sums: scratch of total_tiles int64.
struct ScanJob {
    const int32_t *in;
    int64_t *out;
    int64_t n, tile0;
};
int64_t scan_tiles(int64_t n);
void launch_multi_scan(const ScanJob *jobs_dev, int njobs, int64_t total_tiles, int64_t *tile_sums, hipStream_t s);
// Everything the diff builder needs for one pair of consecutive snapshots (a = t-1, b = t): inputs, scratch, outputs.
// A table of these in device memory lets one launch work on many pairs (blockIdx.y picks the pair).
struct DiffStep {
    const int32_t *col_a, *col_b;
    const int64_t *rp_a, *rp_b;
    const void *x_a, *x_b;
    const float *p_a, *p_b;
    const int32_t *feat_rows;  // rows re-assigned at t (delta-mode loading), or null
    int64_t n_feat_rows;
    // scratch: change-set flags and their prefix sums, the change set as a bit per node, four counts per row and the
    // prefix sums of the last (changed rows), the per-entry flag bits
    int32_t *cflags;
    int64_t *coffs;
    uint64_t *bits;
    int32_t *cnt_ins, *cnt_del, *cnt_ent, *row_flag;
    int64_t *roffs;
    uint64_t *mask_ins, *mask_del, *mask_hit;  // a bit per entry: absent from the other snapshot / source in the change set
    // outputs
    int64_t *ins_ptr, *del_ptr, *ent_ptr;
    int32_t *ins_col, *del_col;
    uint32_t *ent;
    int32_t *rows, *changed;
    int64_t *row_ent;
    float *dY;
    int64_t n_changed;
};
// stage 0: change-set flags; 1: the change set as bits and the per-row counts; 2: every output.  The prefix sums
// between the stages are the caller's.  max_list / max_changed: the largest count of any pair (the grid covers it).
void launch_diff_stage(int stage, const DiffStep *steps_dev, int count, int64_t n, int64_t max_list, int64_t max_changed, int sym,
                       int self_loop, int bf16, int32_t d, hipStream_t s);
// dst[i] = *src_dev[i] for i < count (src_dev: pointer table in device memory)
void launch_gather_i64(const int64_t *const *src_dev, int count, int64_t *dst, hipStream_t s);
void launch_fill_i32(int32_t *p, int64_t n, int32_t v, hipStream_t s);
void launch_feature_flags_compare(const void *x_prev, const void *x_cur, int64_t n, int32_t row_bytes, int32_t *flags,
                                  hipStream_t s);
void launch_compact(const int32_t *flags, const int64_t *offsets, int64_t n, int32_t *list, int32_t *index_of,
                    hipStream_t s);
// canonicalisation of a raw edge list
size_t sort_keys_tmp_bytes(int64_t n);
// stable sort by the key bits [begin_bit, end_bit)
hipError_t sort_keys(void *tmp, size_t tmp_bytes, const uint64_t *in, uint64_t *out, int64_t n, unsigned begin_bit, unsigned end_bit,
                     hipStream_t s);
void launch_make_keys(const int32_t *src, const int32_t *dst, int64_t nnz, int64_t n, uint64_t *keys, int32_t *err,
                      hipStream_t s);
void launch_unique_flags(const uint64_t *keys, int64_t nnz, int64_t n, int32_t *flag, hipStream_t s);
void launch_scatter_unique(const uint64_t *keys, const int32_t *flag, const int64_t *offs, int64_t nnz, int32_t *col,
                           int32_t *rowid, uint64_t *swapped, hipStream_t s);
void launch_low_halves(const uint64_t *keys, int64_t e, int32_t *out, hipStream_t s);
void launch_ptr_from_sorted(const uint64_t *keys, int64_t e, int64_t n, int64_t *ptr, hipStream_t s);
void launch_ptr_from_rowid(const int32_t *rowid, int64_t e, int64_t n, int64_t *ptr, hipStream_t s);
void launch_degree_scales(const int64_t *ptr, int64_t n, int sym, int self_loop, float *q, hipStream_t s);
void launch_long_flags(const int64_t *ptr, int64_t n, int32_t *flag, hipStream_t s);
// keys[v] = (kLongRow + 1 - min(length of row v, kLongRow + 1)) << 32 | v: ascending keys = falling row length
void launch_length_keys(const int64_t *ptr, int64_t n, uint64_t *keys, hipStream_t s);
void launch_scatter_rows(const void *vals, const int32_t *rows, int64_t nrows, int32_t row_bytes, void *x, hipStream_t s);

// ---- kernels_agg.hip
bool agg_width_supported(int32_t d, int bf16);
// out[v] = out_scale[v] * ( self_loop * in_scale[v] X[v] + sum_{e in [ptr[v], ptr[v+1])} in_scale[idx[e]] X[idx[e]] )
// in_scale / out_scale may be null (factor 1); then + bias and relu (AggItem); mask [n,d] (may be null) zeroes the
// output where mask <= 0.
// One launch serves a batch of up to kMaxAggBatch snapshots (blockIdx.y picks the item): the layers above the
// first aggregate every timestep of a window in one go.  launch_aggregate_batch takes every row of at most kLongRow
// entries (all rows of an item with n_long == 0); launch_aggregate_long_batch takes the listed long rows with one
// block each.
void launch_aggregate_batch(const AggBatch &batch, int bf16, int32_t d, int64_t n, int self_loop, hipStream_t s,
                            hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);
void launch_aggregate_long_batch(const AggBatch &batch, int bf16, int32_t d, int self_loop, hipStream_t s);
// both, with the main kernel timed as REINC_K_AGG_FULL; n_rows >= 0: only rows [0, n_rows) of the short-row kernel
// (listed long rows beyond it are still computed)
void aggregate_full_batch(reinc_ctx *ctx, const AggBatch &batch, int bf16, int32_t d, int self_loop, hipStream_t s,
                          int64_t n_rows = -1);
void aggregate_full(reinc_ctx *ctx, const int64_t *ptr, const int32_t *idx, const int32_t *long_rows, int32_t n_long,
                    const void *X, int bf16, int32_t d, int self_loop, const float *in_scale, const float *out_scale,
                    const float *mask, float *out, hipStream_t s, const int32_t *order = nullptr);
// max / min aggregation with contributing source ids (Section 3.2): from scratch, and the incremental step whose
// hub rows with a lost contributor are marked in hub_flags [N] (zeroed by the caller) for the block-per-row kernel;
// block_counts needs one int per 4 rows; *stat_out receives the number of rows aggregated from scratch
void launch_minmax_full(const int64_t *ptr, const int32_t *idx, const int32_t *long_rows, int32_t n_long, const void *X,
                        int bf16, int32_t d, int64_t n, int self_loop, int is_max, float *out, int32_t *contrib, hipStream_t s);
void launch_minmax_incremental(const int32_t *rows, int64_t n_rows, const int32_t *long_rows, int32_t n_long,
                               const int64_t *ent_ptr, const uint32_t *ent, const int32_t *changed, const int64_t *ptr,
                               const int32_t *idx, const void *x_cur, int bf16, int32_t d, int self_loop, int is_max,
                               const float *M_prev, const int32_t *C_prev, float *M_out, int32_t *C_out, int32_t *hub_flags,
                               int32_t *block_counts, int32_t *stat_out, hipStream_t s);
// Eq. 2 over the merged signed delta rows.  rows != null: the listed rows only (in place), row_ent [n_rows + 1] = where
// the entries of the i-th listed row begin; rows == null: every row 0 .. n_rows-1 through ent_ptr, rows without
// entries are copied from S_prev to S_out.  ev_start / ev_stop (optional) are stamped with the kernel's begin and end.
void launch_incremental(const int32_t *rows, const int64_t *row_ent, int64_t n_rows, const int64_t *ent_ptr,
                        const uint32_t *ent, const void *x_prev, int bf16, const float *p_prev, const float *dY, int32_t d,
                        const float *S_prev, float *S_out, const float *q, float *agg_out, hipStream_t s,
                        hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);

// ---- kernels_dense.hip
// out[n,M] = epilogue((row_scale .* A)[n,K] * B[K,M]); B = W (ldw = row stride) or W^T when w_transposed.
// epilogue: + bias, relu, + add[n,M], zero where mask[n,M] <= 0 (each optional)
int launch_gemm_rows(const void *A, int a_bf16, int64_t n, int32_t K, int32_t M, const float *row_scale, const float *W,
                     int w_transposed, int32_t ldw, const float *bias, int relu, const float *add, const float *mask,
                     float *out, hipStream_t s);
// db[j] (+)= sum over the n rows of G[., j]; partial: scratch of column_sums_bytes(M); fixed summation order
uint64_t column_sums_bytes(int32_t M);
void launch_column_sums(const float *G, int64_t n, int32_t M, float *partial, float *db, int accumulate, hipStream_t s);
// x_scale [n] (or null) multiplies the rows of x; h_prev is the recurrent GEMM operand, h_carry the state of the GRU
// carry term z .* h (the stacked model passes the same pointer for both)
void launch_rnn_fused(int lstm, const float *x, const float *x_scale, int64_t n, int32_t d_in, int32_t H, const float *h_prev,
                      const float *h_carry, const float *c_prev, const float *W_i, const float *W_h, const float *b_i,
                      const float *b_h, float *h_out, float *c_out, float *saved, hipStream_t s);
uint64_t reduce_partial_bytes(int64_t n, int32_t K, int32_t M);
// partial[chunk] (+)= (row_scale .* A)^T G over the chunk's rows, with the column sums of G in row K; `accumulate`
// adds to what the slabs hold.  The slab geometry is that of n_geom >= n rows, so that calls over different row
// counts can add into one set of slabs (sized by reduce_partial_bytes(n_geom, K, M)).  launch_reduce_partials
// (with the same n_geom) then does dW[K,M] += sum of slabs, db[M] += sum of rows K.
void launch_gemm_reduce(const float *A, int32_t lda, const float *row_scale, const float *G, int32_t ldg, int64_t n,
                        int64_t n_geom, int32_t K, int32_t M, float *partial, int accumulate, hipStream_t s);
void launch_reduce_partials(const float *partial, int64_t n, int32_t K, int32_t M, float *dW, float *db, hipStream_t s);
void launch_rnn_backward_elem(int lstm, int64_t n, int32_t H, const float *dh, const float *dc, const float *saved,
                              const float *h_prev, const float *c_prev, const float *c_new, float *dgi, float *dgh,
                              float *dh_carry, float *dc_prev, hipStream_t s);
uint64_t loss_partial_bytes();
void launch_mse(const float *h, const float *y, int64_t total, float *partial, float *loss, hipStream_t s);
// dh[i] = d mean((h - y)^2 over the first `counted` elements) / d h[i] for i < total (zero from `counted` on)
void launch_mse_grad(const float *h, const float *y, int64_t counted, int64_t total, float *dh, hipStream_t s);
void launch_fill_f32(float *p, int64_t n, float v, hipStream_t s);
void launch_sgd(float *params, const float *grads, int64_t n, float lr, hipStream_t s);
}  // namespace reinc
