// Node mini-batches (paper Section 4.2, "Rethinking Mini-batch Training"): a set of nodes is selected, the
// computational graphs of those nodes are extracted from every snapshot of the sequence, and that sequence of
// computational graphs is the sample.  Here the extraction runs on the device, from the canonical snapshots a
// context holds, into a second, smaller context that is then driven like any other: its windows slide over the
// whole sequence before the next batch is taken (seq-first), so its aggregate cache serves every window of the
// batch and holds the rows of this batch only.
//
//   F_0 = the batch,  F_k = F_{k-1} and the sources of every edge, of any snapshot, whose target is in F_{k-1};
//   the sub-sequence keeps the nodes F_hops and, of every snapshot, the edges whose target is in F_{hops-1}.
// Numbering of the sub-sequence: batch nodes first, in the order given, then the others by ascending id.
#include <algorithm>
#include <climits>
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

// hop k: the source of an edge whose target was reached in fewer than k hops is reached in at most k.  Levels
// below k are final and levels of k are only ever written as k during this launch, so the order of the threads
// does not matter.
__global__ void batch_expand(const int32_t *rowid, const int32_t *col, int64_t e, int32_t *level, int32_t k)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i >= e) return;
    if (level[rowid[i]] < k) atomicMin(&level[col[i]], k);
}

// flags of the nodes that join the batch nodes in the sub-sequence, and the count of inner nodes (targets kept)
__global__ void batch_member_flags(const int32_t *level, int64_t n, int32_t hops, int32_t *flag, unsigned long long *inner)
{
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v >= n) return;
    const int32_t l = level[v];
    flag[v] = l >= 1 && l <= hops;
    if (l < hops) atomicAdd(inner, 1ull);
}

__global__ void batch_number(const int32_t *flag, const int64_t *offs, int64_t n, int64_t nb, int32_t *new_id, int32_t *node_list)
{
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v >= n || !flag[v]) return;
    const int64_t id = nb + offs[v];
    new_id[v] = int32_t(id);
    node_list[id] = int32_t(v);
}

__global__ void batch_edge_flags(const int32_t *rowid, int64_t e, const int32_t *level, int32_t hops, int32_t *flag)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i < e) flag[i] = level[rowid[i]] < hops;
}

__global__ void batch_edge_compact(const int32_t *rowid, const int32_t *col, int64_t e, const int32_t *flag, const int64_t *offs,
                                   const int32_t *new_id, int32_t *src, int32_t *dst)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i >= e || !flag[i]) return;
    src[offs[i]] = new_id[col[i]];
    dst[offs[i]] = new_id[rowid[i]];
}

__global__ void gather_f32(const float *in, const int32_t *list, int64_t n, float *out)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i < n) out[i] = in[list[i]];
}

// out row i = in row list[i], in 16-byte pieces
__global__ void gather_rows(const uint4 *in, const int32_t *list, int64_t nrows, int32_t chunks, uint4 *out)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i >= nrows * chunks) return;
    const int64_t r = i / chunks;
    out[i] = in[int64_t(list[r]) * chunks + (i - r * chunks)];
}

}  // namespace
}  // namespace reinc

extern "C" {

int reinc_set_loss_rows(reinc_ctx *ctx, int64_t rows)
{
    if (!ctx) return REINC_E_ARG;
    if (rows < 0 || rows > ctx->N()) return ctx->fail(REINC_E_ARG, "loss rows %lld outside [0, %lld]", (long long)rows, (long long)ctx->N());
    ctx->loss_rows = rows == ctx->N() ? 0 : rows;
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
    int32_t *flag = static_cast<int32_t *>(ctx->scratch(uint64_t(n) * 4));
    int64_t *offs = static_cast<int64_t *>(ctx->scratch(uint64_t(n + 1) * 8));
    void *scan_tmp = ctx->scratch(scan_tmp_bytes(n));
    int64_t *counters = static_cast<int64_t *>(ctx->scratch(256));  // [0] inner nodes, [1] (as int32) duplicate flag
    if (!d_nodes || !flag || !offs || !scan_tmp || !counters) {
        ctx->scratch_reset();
        return ctx->fail(REINC_E_NOMEM, "arena exhausted while planning a node batch");
    }
    int32_t *err = reinterpret_cast<int32_t *>(counters + 1);
    REINC_HIP(ctx, hipMemcpy(d_nodes, nodes, size_t(n_batch) * 4, hipMemcpyHostToDevice));
    launch_fill_i32(ctx->batch_level, n, kFar, s);
    launch_fill_i32(ctx->batch_new_id, n, -1, s);
    launch_fill_i32(reinterpret_cast<int32_t *>(counters), 4, 0, s);
    batch_seed<<<blocks_for(n_batch, 256), 256, 0, s>>>(d_nodes, n_batch, ctx->batch_level, ctx->batch_new_id, ctx->batch_nodes, err);
    for (int32_t k = 1; k <= hops; ++k)
        for (const Snapshot &sn : ctx->snaps)
            if (sn.nnz > 0) batch_expand<<<blocks_for(sn.nnz, 256), 256, 0, s>>>(sn.rowid, sn.col, sn.nnz, ctx->batch_level, k);
    batch_member_flags<<<blocks_for(n, 256), 256, 0, s>>>(ctx->batch_level, n, hops, flag, reinterpret_cast<unsigned long long *>(counters));
    launch_scan(flag, offs, n, scan_tmp, s);
    batch_number<<<blocks_for(n, 256), 256, 0, s>>>(flag, offs, n, n_batch, ctx->batch_new_id, ctx->batch_nodes);
    REINC_HIP(ctx, hipGetLastError());
    int64_t joined = 0, host_counters[2] = {0, 0};
    REINC_HIP(ctx, hipMemcpy(&joined, offs + n, 8, hipMemcpyDeviceToHost));
    REINC_HIP(ctx, hipMemcpy(host_counters, counters, 16, hipMemcpyDeviceToHost));
    ctx->scratch_reset();
    if (int32_t(host_counters[1] & 0xffffffff)) return ctx->fail(REINC_E_ARG, "a node is listed twice in the batch");
    ctx->batch_size = n_batch;
    ctx->batch_total = n_batch + joined;
    ctx->batch_hops = hops;
    if (n_nodes_out) *n_nodes_out = ctx->batch_total;
    if (n_inner_out) *n_inner_out = host_counters[0];
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
    const int32_t row_bytes = int32_t(a.dims[0] * ctx->elem_bytes());
    if (row_bytes % 16 != 0) return ctx->fail(REINC_E_UNSUPPORTED, "feature rows of %d bytes", row_bytes);
    int64_t max_e = 1;
    for (const Snapshot &sn : ctx->snaps) max_e = std::max(max_e, sn.nnz);
    ctx->scratch_reset();
    int32_t *flag = static_cast<int32_t *>(ctx->scratch(uint64_t(max_e) * 4));
    int64_t *offs = static_cast<int64_t *>(ctx->scratch(uint64_t(max_e + 1) * 8));
    int32_t *src = static_cast<int32_t *>(ctx->scratch(uint64_t(max_e) * 4));
    int32_t *dst = static_cast<int32_t *>(ctx->scratch(uint64_t(max_e) * 4));
    void *scan_tmp = ctx->scratch(scan_tmp_bytes(max_e));
    if (!flag || !offs || !src || !dst || !scan_tmp) {
        ctx->scratch_reset();
        return ctx->fail(REINC_E_NOMEM, "arena exhausted while extracting a node batch");
    }
    int rc = REINC_OK;
    for (int32_t t = 0; t < a.num_snapshots && rc == REINC_OK; ++t) {
        const Snapshot &sn = ctx->snaps[t];
        int64_t kept = 0;
        if (sn.nnz > 0) {
            batch_edge_flags<<<blocks_for(sn.nnz, 256), 256, 0, s>>>(sn.rowid, sn.nnz, ctx->batch_level, ctx->batch_hops, flag);
            launch_scan(flag, offs, sn.nnz, scan_tmp, s);
            batch_edge_compact<<<blocks_for(sn.nnz, 256), 256, 0, s>>>(sn.rowid, sn.col, sn.nnz, flag, offs, ctx->batch_new_id, src, dst);
            if (hipGetLastError() != hipSuccess || hipMemcpy(&kept, offs + sn.nnz, 8, hipMemcpyDeviceToHost) != hipSuccess) {
                rc = ctx->fail(REINC_E_HIP, "extracting the edges of snapshot %d failed", t);
                break;
            }
        }
        rc = load_edges(child, t, src, dst, kept, true);
        if (rc != REINC_OK) {
            ctx->fail(rc, "batch context: %s", child->err.c_str());
            break;
        }
        Snapshot &cs = child->snaps[t];
        // The degree scales are those of the source graph: a row of the batch graph holds all of a node's in-edges only
        // for the nodes whose aggregate is needed, but the symmetric normalisation also scales by the degree of an
        // edge's source.
        if (cs.q && sn.q) gather_f32<<<blocks_for(nu, 256), 256, 0, s>>>(sn.q, ctx->batch_nodes, nu, cs.q);
        cs.x = child->alloc(uint64_t(nu) * row_bytes);
        if (!cs.x) {
            rc = ctx->fail(REINC_E_NOMEM, "batch context: arena exhausted while storing features of snapshot %d", t);
            break;
        }
        const int32_t chunks = row_bytes / 16;
        gather_rows<<<blocks_for(nu * chunks, 256), 256, 0, s>>>(static_cast<const uint4 *>(sn.x), ctx->batch_nodes, nu, chunks,
                                                                static_cast<uint4 *>(cs.x));
        if (hipGetLastError() != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
            rc = ctx->fail(REINC_E_HIP, "gathering the features of snapshot %d failed", t);
            break;
        }
        cs.feats_loaded = true;
        cs.feats_from_delta = false;
        if (child->has_derived) child->load_after_derived = true;
    }
    ctx->scratch_reset();
    if (rc != REINC_OK) return rc;
    child->loss_rows = ctx->batch_size == nu ? 0 : ctx->batch_size;
    child->local_valid = false;
    return REINC_OK;
}

}  // extern "C"
