// Node mini-batches (paper Section 4.2, "Rethinking Mini-batch Training"): a set of nodes is selected, the
// computational graphs of those nodes are extracted from every snapshot of the sequence, and that sequence of
// computational graphs is the sample.  Here the extraction runs on the device, from the canonical snapshots a
// context holds, into a second, smaller context that is then driven like any other: its windows slide over the
// whole sequence before the next batch is taken (seq-first), so its aggregate cache serves every window of the
// batch and holds the rows of this batch only.
//
//   F_0 = the batch,  F_k = F_{k-1} and the sources of every edge, of any snapshot, whose target is in F_{k-1};
//   the sub-sequence keeps the nodes F_hops and, of every snapshot, the edges whose target is in F_{hops-1}.
// Numbering of the sub-sequence: batch nodes first, in the order given, then the nodes first reached in one hop by
// ascending id, then those first reached in two hops, ...: every F_k is a prefix of the ids, so layer l of an L-layer
// model, which is needed on F_{L-l} only, works on a prefix of the rows.
#include <algorithm>
#include <climits>
#include <cstdlib>
#include <vector>

#include "ctx.h"

using namespace reinc;

namespace reinc {
namespace {

constexpr int32_t kFar = INT_MAX;

inline unsigned blocks_for(int64_t n, int threads) { return unsigned((n + threads - 1) / threads); }

// level 0 for the batch nodes and their new ids; a node listed twice raises the error flag
__global__ void batch_seed(const int32_t *nodes, int64_t nb, int32_t *level, int32_t *new_id, int32_t *node_list, int32_t *err)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i >= nb) return;
    const int32_t v = nodes[i];
    if (atomicExch(&level[v], 0) == 0) atomicExch(err, 1);
    new_id[v] = int32_t(i);
    node_list[i] = v;
}

// flag[(k - 1) * n + v] = node v is first reached in exactly k hops, k = 1 .. hops: the scan of these flags numbers
// the nodes that join the batch by hop count first and by id second
__global__ void batch_level_flags(const int32_t *level, int64_t n, int32_t hops, int32_t *flag)
{
    const int64_t idx = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (idx >= n * hops) return;
    const int64_t k = idx / n;
    flag[idx] = level[idx - k * n] == int32_t(k + 1);
}

// new ids and the node list; counts[k] = nodes first reached in 1 .. k hops, k = 0 .. hops
__global__ void batch_number(const int32_t *level, const int64_t *offs, int64_t n, int32_t hops, int64_t nb, int32_t *new_id,
                             int32_t *node_list, int64_t *counts)
{
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v <= hops) counts[v] = offs[v * n];
    if (v >= n) return;
    const int32_t l = level[v];
    if (l < 1 || l > hops) return;
    const int64_t id = nb + offs[int64_t(l - 1) * n + v];
    new_id[v] = int32_t(id);
    node_list[id] = int32_t(v);
}

// ---- extraction of all snapshots of the sub-sequence in one pass: blockIdx.y (or a key's top bits) picks the snapshot ----
// A batch graph is small (thousands of rows), so one snapshot at a time would be a few dozen launches of almost
// empty kernels per snapshot.  Here every step handles the T snapshots together; the source and the batch context
// are described to the kernels by one table each.
struct MbSrc {
    const int64_t *row_ptr;
    const int32_t *rowid, *col;
    const float *q;
    const void *x;
    int64_t nnz;
};
struct MbDst {
    int64_t *row_ptr, *col_ptr;
    int32_t *col, *rowid, *row, *row_order, *col_order, *long_rows, *long_cols;
    float *q;
    void *x;
};

// hop k: the sources of the rows reached in exactly k - 1 hops are reached in at most k (the rows reached earlier
// were expanded in an earlier hop).  Levels of k - 1 are final and levels are only ever lowered to k during this
// launch, so the order of the threads does not matter.  16 lanes walk one row.
__global__ void mb_expand(const MbSrc *src, int32_t *level, int32_t k, int64_t n)
{
    const int64_t v = (blockIdx.x * int64_t(blockDim.x) + threadIdx.x) >> 4;
    if (v >= n || level[v] != k - 1) return;
    const MbSrc sn = src[blockIdx.y];
    const int64_t end = sn.row_ptr[v + 1];
    for (int64_t i = sn.row_ptr[v] + (threadIdx.x & 15); i < end; i += 16) {
        const int32_t u = sn.col[i];
        if (level[u] > k) atomicMin(&level[u], k);
    }
}

// counts[t * nu + i] = in-edges that row i of the batch graph keeps in snapshot t: all of them if the node's aggregate
// is needed (it was reached in fewer than `hops` hops), none otherwise
__global__ void mb_row_counts(const MbSrc *src, const int32_t *nodes, const int32_t *level, int32_t hops, int64_t nu, int32_t *counts)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i >= nu) return;
    const int32_t v = nodes[i];
    const int64_t *ptr = src[blockIdx.y].row_ptr;
    counts[blockIdx.y * nu + i] = level[v] < hops ? int32_t(ptr[v + 1] - ptr[v]) : 0;
}

// the rows are emitted in the order of their new ids, so the scanned counts are the row pointers already
__global__ void mb_row_ptrs(const MbDst *dst, const int64_t *offs, int64_t nu, int64_t *kbase)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i > nu) return;
    const int64_t t = blockIdx.y, base = offs[t * nu];
    dst[t].row_ptr[i] = offs[t * nu + i] - base;
    if (i == 0) kbase[t] = base;
    if (i == nu && t + 1 == gridDim.y) kbase[t + 1] = offs[t * nu + nu];
}

// keys of the kept edges, snapshot << 2 shift | new source << shift | new target, written in ascending order of
// snapshot and target: 16 lanes copy one row
__global__ void mb_edge_keys(const MbSrc *src, const int32_t *nodes, const int32_t *level, const int32_t *new_id, int32_t hops, int64_t nu,
                             int64_t rows_total, const int64_t *offs, unsigned shift, uint64_t *keys)
{
    const int64_t r = (blockIdx.x * int64_t(blockDim.x) + threadIdx.x) >> 4;
    const int lane = threadIdx.x & 15;
    if (r >= rows_total) return;
    const int64_t t = r / nu, i = r - t * nu;
    const int32_t v = nodes[i];
    if (level[v] >= hops) return;
    const MbSrc sn = src[t];
    const int64_t b = sn.row_ptr[v], len = sn.row_ptr[v + 1] - b, out = offs[r];
    const uint64_t rest = (uint64_t(t) << (2 * shift)) | uint64_t(i);
    for (int64_t e = lane; e < len; e += 16) keys[out + e] = rest | (uint64_t(uint32_t(new_id[sn.col[b + e]])) << shift);
}

// keys in the order of snapshot, source, target -> the row ids of every snapshot's CSC, and the same edges keyed
// snapshot << 2 shift | target << shift | source
__global__ void mb_csc_entries(const uint64_t *keys, int64_t total, unsigned shift, const int64_t *kbase, const MbDst *dst, uint64_t *swapped)
{
    const int64_t j = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (j >= total) return;
    const uint64_t k = keys[j], mask = (uint64_t(1) << shift) - 1, t = k >> (2 * shift), lo = k & mask, hi = (k >> shift) & mask;
    dst[t].row[j - kbase[t]] = int32_t(lo);
    swapped[j] = (t << (2 * shift)) | (lo << shift) | hi;
}

// keys in the order of snapshot, target, source -> the entries of every snapshot's CSR
__global__ void mb_csr_entries(const uint64_t *keys, int64_t total, unsigned shift, const int64_t *kbase, const MbDst *dst)
{
    const int64_t j = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (j >= total) return;
    const uint64_t k = keys[j], mask = (uint64_t(1) << shift) - 1, t = k >> (2 * shift);
    const int64_t local = j - kbase[t];
    dst[t].col[local] = int32_t(k & mask);
    dst[t].rowid[local] = int32_t((k >> shift) & mask);
}

// the column pointers, from the keys in the order of snapshot, source, target
__global__ void mb_col_ptrs(const uint64_t *keys, unsigned shift, const int64_t *kbase, const MbDst *dst, int64_t nu)
{
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v > nu) return;
    const int64_t t = blockIdx.y, begin = kbase[t];
    const uint64_t mask = (uint64_t(1) << shift) - 1;
    int64_t lo = begin, hi = kbase[t + 1];
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (int64_t((keys[mid] >> shift) & mask) < v)
            lo = mid + 1;
        else
            hi = mid;
    }
    dst[t].col_ptr[v] = lo - begin;
}

// Degree scales and features of the batch rows.  The scales are those of the source graph: a row of the batch graph
// holds all of a node's in-edges only for the nodes whose aggregate is needed, but the symmetric normalisation also
// scales by the degree of an edge's source.
__global__ void mb_gather_scales(const MbSrc *src, const MbDst *dst, const int32_t *nodes, int64_t nu)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i < nu) dst[blockIdx.y].q[i] = src[blockIdx.y].q[nodes[i]];
}

// out row i = in row nodes[i], in 16-byte pieces
__global__ void mb_gather_rows(const MbSrc *src, const MbDst *dst, const int32_t *nodes, int64_t nu, int32_t chunks)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i >= nu * chunks) return;
    const int64_t r = i / chunks;
    static_cast<uint4 *>(dst[blockIdx.y].x)[i] = static_cast<const uint4 *>(src[blockIdx.y].x)[int64_t(nodes[r]) * chunks + (i - r * chunks)];
}

// per row (y < T) and per column (y >= T) of every snapshot: the key that orders it by falling length, and whether
// it takes the block-per-row path
__global__ void mb_length_keys(const MbDst *dst, int64_t nu, int32_t T, uint64_t *keys, int32_t *flag)
{
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v >= nu) return;
    const int64_t y = blockIdx.y;
    const int64_t *ptr = y < T ? dst[y].row_ptr : dst[y - T].col_ptr;
    const int64_t full = ptr[v + 1] - ptr[v], len = min(full, int64_t(kLongRow + 1));
    keys[y * nu + v] = (uint64_t(y) << 39) | (uint64_t(kLongRow + 1 - len) << 32) | uint64_t(v);
    flag[y * nu + v] = full > kLongRow;
}

__global__ void mb_orders(const uint64_t *keys, const MbDst *dst, int64_t nu, int32_t T)
{
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v >= nu) return;
    const int64_t y = blockIdx.y;
    int32_t *out = y < T ? dst[y].row_order : dst[y - T].col_order;
    out[v] = int32_t(keys[y * nu + v] & 0xFFFFFFFFu);
}

__global__ void mb_long_lists(const int32_t *flag, const int64_t *offs, const MbDst *dst, int64_t nu, int32_t T, int64_t *n_long)
{
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v >= nu) return;
    const int64_t y = blockIdx.y, base = offs[y * nu];
    int32_t *list = y < T ? dst[y].long_rows : dst[y - T].long_cols;
    if (flag[y * nu + v]) list[offs[y * nu + v] - base] = int32_t(v);
    if (v == nu - 1) n_long[y] = offs[y * nu + nu] - base;
}

// the table of the source snapshots, in scratch memory of ctx (null: no room or the copy failed)
const MbSrc *source_table(reinc_ctx *ctx, int64_t *max_e)
{
    std::vector<MbSrc> host;
    *max_e = 0;
    for (const Snapshot &sn : ctx->snaps) {
        host.push_back(MbSrc{sn.row_ptr, sn.rowid, sn.col, sn.q, sn.x, sn.nnz});
        *max_e = std::max(*max_e, sn.nnz);
    }
    void *dev = ctx->scratch(host.size() * sizeof(MbSrc));
    if (!dev || hipMemcpy(dev, host.data(), host.size() * sizeof(MbSrc), hipMemcpyHostToDevice) != hipSuccess) return nullptr;
    return static_cast<const MbSrc *>(dev);
}

// A layer below the last is restricted to the rows it is needed on when they leave out at least this many bytes of
// its input and output per timestep.  (A first version kept full-height slices for such a layer and ran it timestep
// by timestep, which paid from 150 MB on only; with the slices placed next to each other it always pays.)
// REINC_LAYER_ROWS=<MB> overrides it; a huge value switches the restriction off.
constexpr double layer_rows_threshold = 0.0;

unsigned bits_for(int64_t values)  // bits that hold any number in [0, values)
{
    unsigned bits = 1;
    while ((int64_t(1) << bits) < values) ++bits;
    return bits;
}

}  // namespace
}  // namespace reinc

extern "C" {

int reinc_set_loss_rows(reinc_ctx *ctx, int64_t rows)
{
    if (!ctx) return REINC_E_ARG;
    if (rows < 0 || rows > ctx->N()) return ctx->fail(REINC_E_ARG, "loss rows %lld outside [0, %lld]", (long long)rows, (long long)ctx->N());
    ctx->loss_rows = rows == ctx->N() ? 0 : rows;
    for (int64_t &r : ctx->layer_rows) r = 0;  // (only reinc_batch_load knows which rows the layers below need)
    ctx->hop_rows.clear();
    if (ctx->cache_rows > 0) {                 // cached sums that hold some of the rows only are of no use any more
        const int rc = reinc_cache_clear(ctx);
        if (rc != REINC_OK) return rc;
        ctx->cache_rows = 0;
    }
    ctx->local_valid = false;  // a backward call needs a forward call with these rows first
    return REINC_OK;
}

int reinc_batch_plan(reinc_ctx *ctx, const int32_t *nodes, int64_t n_batch, int32_t hops, int64_t *n_nodes_out, int64_t *n_inner_out)
{
    if (!ctx) return REINC_E_ARG;
    const int64_t n = ctx->N();
    if (!nodes || n_batch <= 0 || n_batch > n) return ctx->fail(REINC_E_ARG, "a batch needs between 1 and %lld nodes", (long long)n);
    if (hops <= 0) hops = ctx->cfg.num_gcn_layers;
    if (hops > 64) return ctx->fail(REINC_E_ARG, "%d hops", hops);
    for (int64_t i = 0; i < n_batch; ++i)
        if (nodes[i] < 0 || nodes[i] >= n) return ctx->fail(REINC_E_ARG, "batch node id %d out of range", nodes[i]);
    for (const Snapshot &sn : ctx->snaps)
        if (!sn.edges_loaded) return ctx->fail(REINC_E_STATE, "every snapshot's edges must be loaded before a batch is planned");
    REINC_HIP(ctx, hipSetDevice(ctx->cfg.device));
    hipStream_t s = nullptr;
    ctx->batch_total = 0;
    if (!ctx->batch_level) {  // three arrays of one int per node, kept for every later plan
        ctx->note_derived();
        ctx->batch_level = static_cast<int32_t *>(ctx->alloc(uint64_t(n) * 4));
        ctx->batch_new_id = static_cast<int32_t *>(ctx->alloc(uint64_t(n) * 4));
        ctx->batch_nodes = static_cast<int32_t *>(ctx->alloc(uint64_t(n) * 4));
        if (!ctx->batch_level || !ctx->batch_new_id || !ctx->batch_nodes) {
            ctx->batch_level = nullptr;
            return ctx->fail(REINC_E_NOMEM, "arena exhausted while planning a node batch");
        }
    }
    ctx->scratch_reset();
    int32_t *d_nodes = static_cast<int32_t *>(ctx->scratch(uint64_t(n_batch) * 4));
    int32_t *flag = static_cast<int32_t *>(ctx->scratch(uint64_t(n) * hops * 4));
    int64_t *offs = static_cast<int64_t *>(ctx->scratch(uint64_t(n * hops + 1) * 8));
    void *scan_tmp = ctx->scratch(scan_tmp_bytes(n * hops));
    int64_t *counters = static_cast<int64_t *>(ctx->scratch(1024));  // [0 .. hops] level counts, [hops + 1] (as int32) duplicate flag
    int64_t max_e = 0;
    const MbSrc *src = source_table(ctx, &max_e);
    if (!d_nodes || !flag || !offs || !scan_tmp || !counters || !src) {
        ctx->scratch_reset();
        return ctx->fail(REINC_E_NOMEM, "arena exhausted while planning a node batch");
    }
    int32_t *err = reinterpret_cast<int32_t *>(counters + hops + 1);
    REINC_HIP(ctx, hipMemcpy(d_nodes, nodes, size_t(n_batch) * 4, hipMemcpyHostToDevice));
    launch_fill_i32(ctx->batch_level, n, kFar, s);
    launch_fill_i32(ctx->batch_new_id, n, -1, s);
    launch_fill_i32(err, 2, 0, s);
    batch_seed<<<blocks_for(n_batch, 256), 256, 0, s>>>(d_nodes, n_batch, ctx->batch_level, ctx->batch_new_id, ctx->batch_nodes, err);
    if (max_e > 0)
        for (int32_t k = 1; k <= hops; ++k)
            mb_expand<<<dim3(blocks_for(n * 16, 256), unsigned(ctx->snaps.size())), 256, 0, s>>>(src, ctx->batch_level, k, n);
    batch_level_flags<<<blocks_for(n * hops, 256), 256, 0, s>>>(ctx->batch_level, n, hops, flag);
    launch_scan(flag, offs, n * hops, scan_tmp, s);
    batch_number<<<blocks_for(std::max<int64_t>(n, hops + 1), 256), 256, 0, s>>>(ctx->batch_level, offs, n, hops, n_batch, ctx->batch_new_id,
                                                                              ctx->batch_nodes, counters);
    REINC_HIP(ctx, hipGetLastError());
    std::vector<int64_t> host_counters(size_t(hops) + 2, 0);
    REINC_HIP(ctx, hipMemcpy(host_counters.data(), counters, size_t(hops + 2) * 8, hipMemcpyDeviceToHost));
    ctx->scratch_reset();
    if (int32_t(host_counters[hops + 1] & 0xffffffff)) return ctx->fail(REINC_E_ARG, "a node is listed twice in the batch");
    ctx->batch_size = n_batch;
    ctx->batch_total = n_batch + host_counters[hops];
    ctx->batch_hops = hops;
    ctx->batch_reach.assign(size_t(hops) + 1, 0);  // |F_k|: the nodes reached in at most k hops are the first |F_k| ids
    for (int32_t k = 0; k <= hops; ++k) ctx->batch_reach[k] = n_batch + host_counters[k];
    if (n_nodes_out) *n_nodes_out = ctx->batch_total;
    if (n_inner_out) *n_inner_out = ctx->batch_reach[hops - 1];
    return REINC_OK;
}

int reinc_batch_node_list(reinc_ctx *ctx, int32_t *out)
{
    if (!ctx) return REINC_E_ARG;
    if (!out) return ctx->fail(REINC_E_ARG, "null output");
    if (ctx->batch_total <= 0) return ctx->fail(REINC_E_STATE, "no node batch has been planned");
    REINC_HIP(ctx, hipSetDevice(ctx->cfg.device));
    REINC_HIP(ctx, hipMemcpy(out, ctx->batch_nodes, size_t(ctx->batch_total) * 4, hipMemcpyDeviceToHost));
    return REINC_OK;
}

int reinc_batch_load(reinc_ctx *ctx, reinc_ctx *child)
{
    if (!ctx || !child) return REINC_E_ARG;
    if (child == ctx) return ctx->fail(REINC_E_ARG, "the batch context must be a different context");
    if (ctx->batch_total <= 0) return ctx->fail(REINC_E_STATE, "no node batch has been planned");
    const reinc_config &a = ctx->cfg, &b = child->cfg;
    if (b.num_nodes != ctx->batch_total || b.num_snapshots != a.num_snapshots || b.dims[0] != a.dims[0] || b.feat_dtype != a.feat_dtype ||
        b.device != a.device || b.agg_kind != a.agg_kind || b.self_loop != a.self_loop)
        return ctx->fail(REINC_E_ARG,
                         "the batch context needs %lld nodes, %d snapshots and the feature width, type, aggregator, self-loop flag and "
                         "device of its source",
                         (long long)ctx->batch_total, a.num_snapshots);
    for (const Snapshot &sn : ctx->snaps)
        if (!sn.edges_loaded || !sn.feats_loaded) return ctx->fail(REINC_E_STATE, "every snapshot must be loaded before a batch is extracted");
    for (const Snapshot &sn : child->snaps)
        if (sn.edges_loaded || sn.feats_loaded) return ctx->fail(REINC_E_STATE, "the batch context already holds snapshots");
    REINC_HIP(ctx, hipSetDevice(a.device));
    hipStream_t s = nullptr;
    const int64_t nu = ctx->batch_total;
    const int32_t T = a.num_snapshots;
    const int32_t row_bytes = int32_t(a.dims[0] * ctx->elem_bytes());
    if (row_bytes % 16 != 0) return ctx->fail(REINC_E_UNSUPPORTED, "feature rows of %d bytes", row_bytes);
    const unsigned shift = node_key_bits(nu), tbits = bits_for(T);
    if (2 * shift + tbits > 64 || 2 * T > 65535)
        return ctx->fail(REINC_E_UNSUPPORTED, "a batch of %lld nodes over %d snapshots", (long long)nu, T);
    const bool scaled = a.agg_kind != REINC_AGG_SUM;
    auto fail = [&](int code, const char *what) {
        ctx->scratch_reset();
        return ctx->fail(code, "extracting a node batch: %s", what);
    };

    // what does not depend on the number of kept edges
    std::vector<MbDst> host_dst(size_t(T), MbDst{});
    for (int32_t t = 0; t < T; ++t) {
        Snapshot &cs = child->snaps[t];
        cs.row_ptr = static_cast<int64_t *>(child->alloc(uint64_t(nu + 1) * 8));
        cs.col_ptr = static_cast<int64_t *>(child->alloc(uint64_t(nu + 1) * 8));
        cs.row_order = static_cast<int32_t *>(child->alloc(uint64_t(nu) * 4));
        cs.col_order = static_cast<int32_t *>(child->alloc(uint64_t(nu) * 4));
        cs.x = child->alloc(uint64_t(nu) * row_bytes);
        if (!cs.row_ptr || !cs.col_ptr || !cs.row_order || !cs.col_order || !cs.x) return fail(REINC_E_NOMEM, "batch context: arena exhausted");
        if (scaled) {
            cs.q = child->q_block + int64_t(t) * nu;
            if (a.agg_kind == REINC_AGG_SYM) cs.p = cs.q;
        }
        host_dst[t] = MbDst{cs.row_ptr, cs.col_ptr, nullptr, nullptr, nullptr, cs.row_order, cs.col_order, nullptr, nullptr, cs.q, cs.x};
    }
    ctx->scratch_reset();
    int64_t max_e = 0;
    const MbSrc *src = source_table(ctx, &max_e);
    MbDst *dst = static_cast<MbDst *>(ctx->scratch(uint64_t(T) * sizeof(MbDst)));
    const int64_t rows_total = int64_t(T) * nu;
    int32_t *counts = static_cast<int32_t *>(ctx->scratch(uint64_t(2 * rows_total) * 4));  // later: the long row / column flags
    int64_t *offs = static_cast<int64_t *>(ctx->scratch(uint64_t(2 * rows_total + 1) * 8));
    void *scan_tmp = ctx->scratch(scan_tmp_bytes(2 * rows_total));
    int64_t *kbase = static_cast<int64_t *>(ctx->scratch(uint64_t(T + 1) * 8));
    int64_t *n_long = static_cast<int64_t *>(ctx->scratch(uint64_t(2 * T) * 8));
    if (!src || !dst || !counts || !offs || !scan_tmp || !kbase || !n_long) return fail(REINC_E_NOMEM, "arena exhausted");
    REINC_HIP(ctx, hipMemcpy(dst, host_dst.data(), size_t(T) * sizeof(MbDst), hipMemcpyHostToDevice));
    const dim3 per_row(blocks_for(nu, 256), unsigned(T)), per_ptr(blocks_for(nu + 1, 256), unsigned(T));
    mb_row_counts<<<per_row, 256, 0, s>>>(src, ctx->batch_nodes, ctx->batch_level, ctx->batch_hops, nu, counts);
    launch_scan(counts, offs, rows_total, scan_tmp, s);
    mb_row_ptrs<<<per_ptr, 256, 0, s>>>(dst, offs, nu, kbase);
    if (scaled) mb_gather_scales<<<per_row, 256, 0, s>>>(src, dst, ctx->batch_nodes, nu);
    const int32_t chunks = row_bytes / 16;
    mb_gather_rows<<<dim3(blocks_for(nu * chunks, 256), unsigned(T)), 256, 0, s>>>(src, dst, ctx->batch_nodes, nu, chunks);
    REINC_HIP(ctx, hipGetLastError());
    std::vector<int64_t> host_kbase(size_t(T) + 1, 0);
    REINC_HIP(ctx, hipMemcpy(host_kbase.data(), kbase, size_t(T + 1) * 8, hipMemcpyDeviceToHost));  // (waits for the device)

    // the edge arrays, now that their sizes are known; a list of long rows cannot be longer than edges / (kLongRow + 1)
    const int64_t total = host_kbase[T];
    for (int32_t t = 0; t < T; ++t) {
        Snapshot &cs = child->snaps[t];
        const int64_t kept = host_kbase[t + 1] - host_kbase[t];
        const uint64_t ee = uint64_t(std::max<int64_t>(kept, 1)), longs = uint64_t(kept / (kLongRow + 1) + 1);
        cs.col = static_cast<int32_t *>(child->alloc(ee * 4));
        cs.rowid = static_cast<int32_t *>(child->alloc(ee * 4));
        cs.row = static_cast<int32_t *>(child->alloc(ee * 4));
        cs.long_rows = static_cast<int32_t *>(child->alloc(longs * 4));
        cs.long_cols = static_cast<int32_t *>(child->alloc(longs * 4));
        if (!cs.col || !cs.rowid || !cs.row || !cs.long_rows || !cs.long_cols) return fail(REINC_E_NOMEM, "batch context: arena exhausted");
        cs.nnz = kept;
        host_dst[t].col = cs.col;
        host_dst[t].rowid = cs.rowid;
        host_dst[t].row = cs.row;
        host_dst[t].long_rows = cs.long_rows;
        host_dst[t].long_cols = cs.long_cols;
    }
    const int64_t n_keys = std::max<int64_t>(std::max(total, 2 * rows_total), 1);
    uint64_t *keys0 = static_cast<uint64_t *>(ctx->scratch(uint64_t(n_keys) * 8));
    uint64_t *keys1 = static_cast<uint64_t *>(ctx->scratch(uint64_t(n_keys) * 8));
    const size_t sort_bytes = sort_keys_tmp_bytes(n_keys);
    void *sort_tmp = ctx->scratch(sort_bytes);
    if (!keys0 || !keys1 || !sort_tmp) return fail(REINC_E_NOMEM, "arena exhausted");
    REINC_HIP(ctx, hipMemcpy(dst, host_dst.data(), size_t(T) * sizeof(MbDst), hipMemcpyHostToDevice));
    if (total > 0) {
        mb_edge_keys<<<blocks_for(rows_total * 16, 256), 256, 0, s>>>(src, ctx->batch_nodes, ctx->batch_level, ctx->batch_new_id, ctx->batch_hops,
                                                                      nu, rows_total, offs, shift, keys0);
        // Two stable sorts by the snapshot and one endpoint each.  The keys are written in the order of snapshot and
        // target; sorted by snapshot and source they are the CSC, with the targets of a column ascending; re-keyed
        // and sorted by snapshot and target they are the CSR, with the sources of a row ascending.
        REINC_HIP(ctx, sort_keys(sort_tmp, sort_bytes, keys0, keys1, total, shift, 2 * shift + tbits, s));
    }
    mb_col_ptrs<<<per_ptr, 256, 0, s>>>(keys1, shift, kbase, dst, nu);
    if (total > 0) {
        mb_csc_entries<<<blocks_for(total, 256), 256, 0, s>>>(keys1, total, shift, kbase, dst, keys0);
        REINC_HIP(ctx, sort_keys(sort_tmp, sort_bytes, keys0, keys1, total, shift, 2 * shift + tbits, s));
        mb_csr_entries<<<blocks_for(total, 256), 256, 0, s>>>(keys1, total, shift, kbase, dst);
    }
    // rows and columns by falling length (the keys are written in ascending order of snapshot and node and the sort
    // is stable: the length bits and the snapshot bits suffice), and the lists of long rows and columns
    const dim3 per_side(blocks_for(nu, 256), unsigned(2 * T));
    mb_length_keys<<<per_side, 256, 0, s>>>(dst, nu, T, keys0, counts);
    REINC_HIP(ctx, sort_keys(sort_tmp, sort_bytes, keys0, keys1, 2 * rows_total, 32, 39 + bits_for(2 * T), s));
    mb_orders<<<per_side, 256, 0, s>>>(keys1, dst, nu, T);
    launch_scan(counts, offs, 2 * rows_total, scan_tmp, s);
    mb_long_lists<<<per_side, 256, 0, s>>>(counts, offs, dst, nu, T, n_long);
    REINC_HIP(ctx, hipGetLastError());
    std::vector<int64_t> host_long(size_t(2 * T), 0);
    REINC_HIP(ctx, hipMemcpy(host_long.data(), n_long, size_t(2 * T) * 8, hipMemcpyDeviceToHost));  // (waits for the device)
    ctx->scratch_reset();
    for (int32_t t = 0; t < T; ++t) {
        Snapshot &cs = child->snaps[t];
        cs.n_long_rows = int32_t(host_long[t]);
        cs.n_long_cols = int32_t(host_long[T + t]);
        cs.edges_loaded = true;
        cs.feats_loaded = true;
        cs.feats_from_delta = false;
    }
    if (child->has_derived) child->load_after_derived = true;
    child->loss_rows = ctx->batch_size == nu ? 0 : ctx->batch_size;
    // layer l of the batch context's L layers is needed on the nodes within L - l hops of the batch: the first ids
    const int32_t Lc = b.num_gcn_layers;
    const char *env = std::getenv("REINC_LAYER_ROWS");  // a number of MB: see layer_rows_threshold
    const double threshold = env ? std::atof(env) * 1e6 : layer_rows_threshold;
    for (int32_t l = 1; l <= REINC_MAX_GCN_LAYERS; ++l) {
        const int32_t k = Lc - l;
        child->layer_rows[l] = 0;
        if (l >= Lc || k > ctx->batch_hops || ctx->batch_reach[k] >= nu) continue;
        const double saved = double(nu - ctx->batch_reach[k]) * (b.dims[l - 1] + b.dims[l]) * 4.0;
        if (saved >= threshold) child->layer_rows[l] = ctx->batch_reach[k];
    }
    child->cache_rows = child->rows_of_layer(1) < nu ? child->rows_of_layer(1) : 0;  // (its cache is still empty)
    child->hop_rows.clear();
    // (the integrated model's rows per timestep, under the same threshold: its last timestep leaves out all but the batch)
    if (child->loss_rows > 0 && double(nu - ctx->batch_size) * (b.dims[0] + b.rnn_hidden) * 4.0 >= threshold)
        child->hop_rows = ctx->batch_reach;
    child->local_valid = false;
    return REINC_OK;
}

}  // extern "C"
