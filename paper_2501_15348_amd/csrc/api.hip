// C-ABI entry points: context, snapshot store, delta builder, aggregation primitives.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>

#include "ctx.h"

using namespace reinc;

namespace {

hipStream_t as_stream(void *s) { return static_cast<hipStream_t>(s); }

int check_t(reinc_ctx *ctx, int32_t t)
{
    if (t < 0 || t >= ctx->cfg.num_snapshots)
        return ctx->fail(REINC_E_ARG, "snapshot index %d outside [0, %d)", t, ctx->cfg.num_snapshots);
    return REINC_OK;
}

template <typename T>
int upload(reinc_ctx *ctx, T **dst, const T *host, int64_t count, const char *what)
{
    *dst = static_cast<T *>(ctx->alloc(uint64_t(std::max<int64_t>(count, 1)) * sizeof(T)));
    if (!*dst) return ctx->fail(REINC_E_NOMEM, "arena exhausted while storing %s (%lld bytes)", what, (long long)(count * sizeof(T)));
    if (count > 0) REINC_HIP(ctx, hipMemcpy(*dst, host, size_t(count) * sizeof(T), hipMemcpyHostToDevice));
    return REINC_OK;
}

template <typename T>
int read_back(reinc_ctx *ctx, T *host, const T *dev, int64_t count)
{
    if (host && count > 0) REINC_HIP(ctx, hipMemcpy(host, dev, size_t(count) * sizeof(T), hipMemcpyDeviceToHost));
    return REINC_OK;
}

float scale_of(int agg, bool target_side, int64_t deg)
{
    if (agg == REINC_AGG_SUM) return 1.0f;
    if (agg == REINC_AGG_MEAN && !target_side) return 1.0f;
    if (deg <= 0) return 0.0f;
    if (agg == REINC_AGG_MEAN) return float(1.0 / double(deg));
    return float(1.0 / std::sqrt(double(deg)));
}

}  // namespace

extern "C" {

const char *reinc_version(void) { return "reinc-hip 0.1 (gfx950)"; }

int reinc_create(reinc_ctx **out, const reinc_config *cfg)
{
    if (!out || !cfg) return REINC_E_ARG;
    *out = nullptr;
    if (cfg->struct_size != sizeof(reinc_config)) return REINC_E_ARG;
    reinc_ctx *ctx = new (std::nothrow) reinc_ctx();
    if (!ctx) return REINC_E_NOMEM;
    *out = ctx;  // returned even on failure so that reinc_last_error() can explain; the caller destroys it
    ctx->cfg = *cfg;
    const reinc_config &c = ctx->cfg;
    if (c.num_nodes <= 0 || c.num_nodes > kMaxNodes) return ctx->fail(REINC_E_ARG, "num_nodes must be in [1, 2^30]");
    if (c.num_snapshots <= 0) return ctx->fail(REINC_E_ARG, "num_snapshots must be positive");
    if (c.num_gcn_layers < 1 || c.num_gcn_layers > REINC_MAX_GCN_LAYERS)
        return ctx->fail(REINC_E_ARG, "num_gcn_layers must be in [1, %d]", REINC_MAX_GCN_LAYERS);
    for (int l = 0; l <= c.num_gcn_layers; ++l)
        if (c.dims[l] <= 0) return ctx->fail(REINC_E_ARG, "dims[%d] must be positive", l);
    if (c.rnn_kind != REINC_RNN_GRU && c.rnn_kind != REINC_RNN_LSTM) return ctx->fail(REINC_E_ARG, "bad rnn_kind");
    if (c.rnn_hidden <= 0) return ctx->fail(REINC_E_ARG, "rnn_hidden must be positive");
    if (c.agg_kind < REINC_AGG_SUM || c.agg_kind > REINC_AGG_SYM) return ctx->fail(REINC_E_ARG, "bad agg_kind");
    if (c.self_loop != 0 && c.self_loop != 1) return ctx->fail(REINC_E_ARG, "self_loop must be 0 or 1");
    if (c.feat_dtype != REINC_F32 && c.feat_dtype != REINC_BF16) return ctx->fail(REINC_E_ARG, "bad feat_dtype");
    if (!agg_width_supported(c.dims[0], c.feat_dtype == REINC_BF16))
        return ctx->fail(REINC_E_UNSUPPORTED, "feature row of %d elements: row bytes must be a power of two in [16, 1024]",
                         c.dims[0]);
    if (!c.arena || (reinterpret_cast<uintptr_t>(c.arena) & 255)) return ctx->fail(REINC_E_ARG, "arena must be a 256-byte aligned device pointer");
    REINC_HIP(ctx, hipSetDevice(c.device));
    ctx->base = static_cast<char *>(c.arena);
    ctx->size = c.arena_bytes & ~uint64_t(255);
    ctx->bottom = 0;
    ctx->top = ctx->size;
    ctx->snaps.resize(c.num_snapshots);
    ctx->deltas.resize(c.num_snapshots);
    ctx->gcache.assign(c.num_snapshots, nullptr);
    if (const char *e = std::getenv("REINC_BATCH")) ctx->max_batch = std::min(std::max(std::atoi(e), 1), int(kMaxAggBatch));
    if (c.agg_kind != REINC_AGG_SUM) {
        ctx->q_block = static_cast<float *>(ctx->alloc(uint64_t(c.num_snapshots) * uint64_t(c.num_nodes) * 4));
        if (!ctx->q_block) return ctx->fail(REINC_E_NOMEM, "arena exhausted: no room for the degree scales");
    }
    return static_scratch_init(ctx);
}

int reinc_destroy(reinc_ctx *ctx)
{
    if (ctx) {
        for (hipEvent_t e : ctx->prof_events) (void)hipEventDestroy(e);
    }
    delete ctx;
    return REINC_OK;
}

const char *reinc_last_error(const reinc_ctx *ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int reinc_arena_free_bytes(const reinc_ctx *ctx, uint64_t *out)
{
    if (!ctx || !out) return REINC_E_ARG;
    *out = ctx->top - ctx->bottom;
    return REINC_OK;
}

// ------------------------------------------------------------------------------------------------ loading

int reinc_load_edges(reinc_ctx *ctx, int32_t t, const int32_t *src, const int32_t *dst, int64_t nnz, int on_device)
{
    if (!ctx) return REINC_E_ARG;
    return reinc::load_edges(ctx, t, src, dst, nnz, on_device != 0);
}

// Scratch of the device-side canonicalisation of one snapshot of at most m raw edges (n nodes).
struct LoadScratch {
    int32_t *d_src, *d_dst;
    uint64_t *keys0, *keys1;
    int32_t *flag, *flag2;
    int64_t *offs, *offs2;
    int64_t *counts;  // small: totals gathered for one copy to the host
    void *sort_tmp, *scan_tmp;
    size_t sort_bytes;
    bool ok;
};

static LoadScratch load_scratch(reinc_ctx *ctx, int64_t m, int64_t n, bool raw_lists)
{
    LoadScratch w{};
    const int64_t mm = std::max(std::max<int64_t>(m, 1), n);  // (the key arrays also serve the per-node sort by row length)
    if (raw_lists) {
        w.d_src = static_cast<int32_t *>(ctx->scratch(uint64_t(std::max<int64_t>(m, 1)) * 4));
        w.d_dst = static_cast<int32_t *>(ctx->scratch(uint64_t(std::max<int64_t>(m, 1)) * 4));
    }
    w.keys0 = static_cast<uint64_t *>(ctx->scratch(uint64_t(mm) * 8));
    w.keys1 = static_cast<uint64_t *>(ctx->scratch(uint64_t(mm) * 8));
    w.flag = static_cast<int32_t *>(ctx->scratch(uint64_t(mm) * 4));
    w.offs = static_cast<int64_t *>(ctx->scratch(uint64_t(mm + 1) * 8));
    w.flag2 = static_cast<int32_t *>(ctx->scratch(uint64_t(n) * 4));
    w.offs2 = static_cast<int64_t *>(ctx->scratch(uint64_t(n + 1) * 8));
    w.counts = static_cast<int64_t *>(ctx->scratch(256));
    w.sort_bytes = sort_keys_tmp_bytes(mm);
    w.sort_tmp = ctx->scratch(w.sort_bytes);
    w.scan_tmp = ctx->scratch(2 * scan_tmp_bytes(mm));
    w.ok = (!raw_lists || (w.d_src && w.d_dst)) && w.keys0 && w.keys1 && w.flag && w.offs && w.flag2 && w.offs2 && w.counts &&
           w.sort_tmp && w.scan_tmp;
    return w;
}

static unsigned node_bits_of(int64_t n)
{
    unsigned bits = 1;
    while ((int64_t(1) << bits) <= n) ++bits;  // the sentinel row id n must sort correctly too
    return bits;
}

extern "C++" unsigned reinc::node_key_bits(int64_t n) { return node_bits_of(n); }

// The rest of a snapshot once its e canonical edges are known: sn.col / sn.rowid hold the CSR entries (allocated and
// filled by the caller), w.keys0 the same edges in the same order keyed by source (source << 32 | target).  Builds
// the row pointers, the CSC, the degree scales, the row / column orders by falling length and the lists of long rows /
// columns.  Waits for the device.
static int finish_snapshot(reinc_ctx *ctx, int32_t t, int64_t e, const LoadScratch &w, uint64_t mark, hipStream_t s)
{
    Snapshot &sn = ctx->snaps[t];
    const int64_t n = ctx->N();
    const unsigned node_bits = node_bits_of(n);
    auto fail_nomem = [&](const char *what) {
        ctx->bottom = mark;
        ctx->scratch_reset();
        sn = Snapshot();
        return ctx->fail(REINC_E_NOMEM, "arena exhausted while canonicalising snapshot %d: %s", t, what);
    };
    launch_ptr_from_rowid(sn.rowid, e, n, sn.row_ptr, s);
    // (w.keys0 is in the CSR's order, ascending by target within a source, and the sort is stable: the source bits suffice)
    REINC_HIP(ctx, sort_keys(w.sort_tmp, w.sort_bytes, w.keys0, w.keys1, e, 32, 32 + node_bits, s));
    launch_low_halves(w.keys1, e, sn.row, s);
    launch_ptr_from_sorted(w.keys1, e, n, sn.col_ptr, s);
    const int agg = ctx->cfg.agg_kind;
    if (agg != REINC_AGG_SUM) {
        sn.q = ctx->q_block + int64_t(t) * n;  // one [T, N] block: the scales of consecutive snapshots are adjacent
        launch_degree_scales(sn.row_ptr, n, agg == REINC_AGG_SYM, ctx->cfg.self_loop, sn.q, s);
        if (agg == REINC_AGG_SYM) sn.p = sn.q;  // same numbers on both sides
    }
    // rows and columns by falling length: the order in which the group-per-row aggregation kernel takes them
    sn.row_order = static_cast<int32_t *>(ctx->alloc(uint64_t(n) * 4));
    sn.col_order = static_cast<int32_t *>(ctx->alloc(uint64_t(n) * 4));
    if (!sn.row_order || !sn.col_order) return fail_nomem("row order lists");
    for (int side = 0; side < 2; ++side) {
        launch_length_keys(side == 0 ? sn.row_ptr : sn.col_ptr, n, w.keys0, s);
        // (the keys are ascending in their low halves, the node ids, and the sort is stable: only the seven bits of the
        // capped length need sorting)
        REINC_HIP(ctx, sort_keys(w.sort_tmp, w.sort_bytes, w.keys0, w.keys1, n, 32, 32 + 7, s));
        launch_low_halves(w.keys1, n, side == 0 ? sn.row_order : sn.col_order, s);
    }
    // rows / columns that take the block-per-row aggregation path: both lists are sized by one copy to the host
    char *scan_tmp2 = static_cast<char *>(w.scan_tmp) + scan_tmp_bytes(n);
    launch_long_flags(sn.row_ptr, n, w.flag, s);
    launch_scan(w.flag, w.offs, n, w.scan_tmp, s);
    launch_long_flags(sn.col_ptr, n, w.flag2, s);
    launch_scan(w.flag2, w.offs2, n, scan_tmp2, s);
    int64_t cnt[2] = {0, 0};
    REINC_HIP(ctx, hipMemcpyAsync(&cnt[0], w.offs + n, 8, hipMemcpyDeviceToHost, s));
    REINC_HIP(ctx, hipMemcpyAsync(&cnt[1], w.offs2 + n, 8, hipMemcpyDeviceToHost, s));
    REINC_HIP(ctx, hipStreamSynchronize(s));
    sn.long_rows = static_cast<int32_t *>(ctx->alloc(uint64_t(std::max<int64_t>(cnt[0], 1)) * 4));
    sn.long_cols = static_cast<int32_t *>(ctx->alloc(uint64_t(std::max<int64_t>(cnt[1], 1)) * 4));
    if (!sn.long_rows || !sn.long_cols) return fail_nomem("long row lists");
    launch_compact(w.flag, w.offs, n, sn.long_rows, nullptr, s);
    launch_compact(w.flag2, w.offs2, n, sn.long_cols, nullptr, s);
    sn.n_long_rows = int32_t(cnt[0]);
    sn.n_long_cols = int32_t(cnt[1]);
    REINC_HIP(ctx, hipGetLastError());
    REINC_HIP(ctx, hipStreamSynchronize(s));
    sn.nnz = e;
    sn.edges_loaded = true;
    if (ctx->has_derived) ctx->load_after_derived = true;
    return REINC_OK;
}

static int alloc_snapshot_arrays(reinc_ctx *ctx, Snapshot &sn, int64_t e)
{
    const int64_t n = ctx->N();
    const uint64_t ee = uint64_t(std::max<int64_t>(e, 1));
    sn.row_ptr = static_cast<int64_t *>(ctx->alloc(uint64_t(n + 1) * 8));
    sn.col = static_cast<int32_t *>(ctx->alloc(ee * 4));
    sn.rowid = static_cast<int32_t *>(ctx->alloc(ee * 4));
    sn.col_ptr = static_cast<int64_t *>(ctx->alloc(uint64_t(n + 1) * 8));
    sn.row = static_cast<int32_t *>(ctx->alloc(ee * 4));
    return sn.row_ptr && sn.col && sn.rowid && sn.col_ptr && sn.row;
}

extern "C++" int reinc::load_edges(reinc_ctx *ctx, int32_t t, const int32_t *src, const int32_t *dst, int64_t nnz, bool on_device)
{
    REINC_TRY(check_t(ctx, t));
    if (nnz < 0 || (nnz > 0 && (!src || !dst))) return ctx->fail(REINC_E_ARG, "null edge arrays");
    Snapshot &sn = ctx->snaps[t];
    if (sn.edges_loaded) return ctx->fail(REINC_E_STATE, "edges of snapshot %d already loaded", t);
    const int64_t n = ctx->N();
    REINC_HIP(ctx, hipSetDevice(ctx->cfg.device));
    hipStream_t s = nullptr;
    // the raw list goes to scratch; everything else happens on the device
    ctx->scratch_reset();
    const uint64_t mark = ctx->bottom;
    auto fail_nomem = [&](const char *what) {
        ctx->bottom = mark;
        ctx->scratch_reset();
        sn = Snapshot();
        return ctx->fail(REINC_E_NOMEM, "arena exhausted while canonicalising snapshot %d: %s", t, what);
    };
    const LoadScratch w = load_scratch(ctx, nnz, n, true);
    int32_t *err = reinterpret_cast<int32_t *>(w.counts);
    if (!w.ok) return fail_nomem("scratch");
    if (nnz > 0) {
        const hipMemcpyKind kind = on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
        REINC_HIP(ctx, hipMemcpy(w.d_src, src, size_t(nnz) * 4, kind));
        REINC_HIP(ctx, hipMemcpy(w.d_dst, dst, size_t(nnz) * 4, kind));
    }
    launch_fill_i32(err, 1, 0, s);
    launch_make_keys(w.d_src, w.d_dst, nnz, n, w.keys0, err, s);
    REINC_HIP(ctx, sort_keys(w.sort_tmp, w.sort_bytes, w.keys0, w.keys1, nnz, 0, 32 + node_bits_of(n), s));
    launch_unique_flags(w.keys1, nnz, n, w.flag, s);
    launch_scan(w.flag, w.offs, nnz, w.scan_tmp, s);
    int64_t e = 0;
    int32_t bad = 0;
    REINC_HIP(ctx, hipMemcpy(&e, w.offs + std::max<int64_t>(nnz, 0), 8, hipMemcpyDeviceToHost));
    REINC_HIP(ctx, hipMemcpy(&bad, err, 4, hipMemcpyDeviceToHost));
    if (bad) {
        ctx->scratch_reset();
        return ctx->fail(REINC_E_ARG, "snapshot %d: an edge endpoint is outside [0, %lld)", t, (long long)n);
    }
    if (!alloc_snapshot_arrays(ctx, sn, e)) return fail_nomem("CSR / CSC");
    // CSR by destination from the sorted unique keys; the same edges keyed by source give the CSC
    launch_scatter_unique(w.keys1, w.flag, w.offs, nnz, sn.col, sn.rowid, w.keys0, s);
    REINC_TRY(finish_snapshot(ctx, t, e, w, mark, s));
    ctx->scratch_reset();
    return REINC_OK;
}

int reinc_load_features_full(reinc_ctx *ctx, int32_t t, const void *X, int on_device)
{
    if (!ctx) return REINC_E_ARG;
    REINC_TRY(check_t(ctx, t));
    if (!X) return ctx->fail(REINC_E_ARG, "null feature matrix");
    Snapshot &sn = ctx->snaps[t];
    if (sn.feats_loaded) return ctx->fail(REINC_E_STATE, "features of snapshot %d already loaded", t);
    REINC_HIP(ctx, hipSetDevice(ctx->cfg.device));
    const uint64_t bytes = uint64_t(ctx->N()) * ctx->cfg.dims[0] * ctx->elem_bytes();
    sn.x = ctx->alloc(bytes);
    if (!sn.x) return ctx->fail(REINC_E_NOMEM, "arena exhausted while storing features of snapshot %d", t);
    REINC_HIP(ctx, hipMemcpy(sn.x, X, bytes, on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice));
    REINC_HIP(ctx, hipDeviceSynchronize());
    sn.feats_loaded = true;
    sn.feats_from_delta = false;
    if (ctx->has_derived) ctx->load_after_derived = true;
    return REINC_OK;
}

int reinc_load_features_delta(reinc_ctx *ctx, int32_t t, const int32_t *rows, int64_t nrows, const void *vals)
{
    if (!ctx) return REINC_E_ARG;
    REINC_TRY(check_t(ctx, t));
    if (t == 0) return ctx->fail(REINC_E_ARG, "snapshot 0 has no predecessor: load it in full");
    if (nrows < 0 || (nrows > 0 && (!rows || !vals))) return ctx->fail(REINC_E_ARG, "null row list or values");
    Snapshot &sn = ctx->snaps[t];
    const Snapshot &pv = ctx->snaps[t - 1];
    if (sn.feats_loaded) return ctx->fail(REINC_E_STATE, "features of snapshot %d already loaded", t);
    if (!pv.feats_loaded) return ctx->fail(REINC_E_STATE, "features of snapshot %d are needed first", t - 1);
    for (int64_t i = 0; i < nrows; ++i) {
        if (rows[i] < 0 || rows[i] >= ctx->N()) return ctx->fail(REINC_E_ARG, "feature row id %d out of range", rows[i]);
        if (i && rows[i] <= rows[i - 1]) return ctx->fail(REINC_E_ARG, "feature row ids must be ascending and unique");
    }
    REINC_HIP(ctx, hipSetDevice(ctx->cfg.device));
    const uint64_t row_bytes = uint64_t(ctx->cfg.dims[0]) * ctx->elem_bytes();
    sn.x = ctx->alloc(uint64_t(ctx->N()) * row_bytes);
    if (!sn.x) return ctx->fail(REINC_E_NOMEM, "arena exhausted while storing features of snapshot %d", t);
    REINC_HIP(ctx, hipMemcpy(sn.x, pv.x, uint64_t(ctx->N()) * row_bytes, hipMemcpyDeviceToDevice));
    REINC_TRY(upload(ctx, &sn.feat_rows, rows, nrows, "feature row ids"));
    // the changed rows travel as one block into scratch and are scattered by a kernel
    ctx->scratch_reset();
    void *staged = ctx->scratch(uint64_t(std::max<int64_t>(nrows, 1)) * row_bytes);
    if (!staged) return ctx->fail(REINC_E_NOMEM, "arena exhausted while staging the feature rows of snapshot %d", t);
    if (nrows > 0) {
        REINC_HIP(ctx, hipMemcpy(staged, vals, uint64_t(nrows) * row_bytes, hipMemcpyHostToDevice));
        launch_scatter_rows(staged, sn.feat_rows, nrows, int32_t(row_bytes), sn.x, nullptr);
        REINC_HIP(ctx, hipGetLastError());
    }
    sn.n_feat_rows = nrows;
    REINC_HIP(ctx, hipDeviceSynchronize());
    ctx->scratch_reset();
    sn.feats_loaded = true;
    sn.feats_from_delta = true;
    if (ctx->has_derived) ctx->load_after_derived = true;
    return REINC_OK;
}

// ------------------------------------------------------------------------------------------------ deltas

// Scratch one step needs while its deltas are being built (bytes, with the allocator's rounding).
static uint64_t diff_mask_bytes(int64_t n, int64_t nnz) { return 8 * uint64_t(nnz / 64 + n / 16 + 4); }  // (64-bit words, one spare per block of at least 16 rows)

static uint64_t step_scratch_bytes(int64_t n, int64_t na, int64_t nb)
{
    auto r = [](int64_t count, int64_t elem) { return (uint64_t(std::max<int64_t>(count, 1)) * elem + 255) & ~uint64_t(255); };
    return 5 * r(n, 4) + 2 * r(n + 1, 8) + r((n + 63) / 64, 8) + r(diff_mask_bytes(n, na), 1) + 2 * r(diff_mask_bytes(n, nb), 1);
}

// Builds the deltas of a group of steps.  Every stage runs for all steps of the group before the next stage begins,
// all prefix sums of a stage are one launch, and the host waits twice per group (for the sizes of the outputs, and at
// the end): on small graphs a step's kernels last microseconds, and step-by-step building was bound by launches and
// round trips to the host.
static int build_group(reinc_ctx *ctx, const std::vector<int32_t> &steps, hipStream_t s)
{
    const int64_t n = ctx->N();
    const int32_t d = ctx->cfg.dims[0];
    const int bf16 = ctx->cfg.feat_dtype == REINC_BF16;
    const int G = int(steps.size());
    if (G == 0) return REINC_OK;
    ctx->scratch_reset();
    ctx->note_derived();
    const uint64_t mark = ctx->bottom;
    auto nomem = [&](const char *what) {
        ctx->bottom = mark;
        ctx->scratch_reset();
        for (int32_t t : steps) ctx->deltas[t] = Delta();
        return ctx->fail(REINC_E_NOMEM, "arena exhausted in build_deltas(%d..%d): %s", steps.front(), steps.back(), what);
    };
    auto i32s = [&](int64_t c) { return static_cast<int32_t *>(ctx->scratch(uint64_t(std::max<int64_t>(c, 1)) * 4)); };
    auto i64s = [&](int64_t c) { return static_cast<int64_t *>(ctx->scratch(uint64_t(std::max<int64_t>(c, 1)) * 8)); };
    // the per-step table for the batched stage kernels: inputs, scratch, and the row pointers of the outputs
    std::vector<DiffStep> table(G);
    int64_t max_list = 0;
    bool compare_features = false, ok = true;
    for (int g = 0; g < G; ++g) {
        const Snapshot &a = ctx->snaps[steps[g] - 1], &b = ctx->snaps[steps[g]];
        Delta &dl = ctx->deltas[steps[g]];
        DiffStep &st = table[g];
        st = DiffStep{};
        st.col_a = a.col, st.col_b = b.col, st.rp_a = a.row_ptr, st.rp_b = b.row_ptr;
        st.x_a = a.x, st.x_b = b.x, st.p_a = a.p, st.p_b = b.p;
        st.feat_rows = b.feats_from_delta ? b.feat_rows : nullptr;
        st.n_feat_rows = b.feats_from_delta ? b.n_feat_rows : 0;
        st.cflags = i32s(n), st.cnt_ins = i32s(n), st.cnt_del = i32s(n), st.cnt_ent = i32s(n), st.row_flag = i32s(n);
        st.coffs = i64s(n + 1), st.roffs = i64s(n + 1);
        st.bits = reinterpret_cast<uint64_t *>(i64s((n + 63) / 64));
        st.mask_del = static_cast<uint64_t *>(ctx->scratch(diff_mask_bytes(n, a.nnz)));
        st.mask_ins = static_cast<uint64_t *>(ctx->scratch(diff_mask_bytes(n, b.nnz)));
        st.mask_hit = static_cast<uint64_t *>(ctx->scratch(diff_mask_bytes(n, b.nnz)));
        dl.ins_ptr = static_cast<int64_t *>(ctx->alloc(uint64_t(n + 1) * 8));
        dl.del_ptr = static_cast<int64_t *>(ctx->alloc(uint64_t(n + 1) * 8));
        dl.ent_ptr = static_cast<int64_t *>(ctx->alloc(uint64_t(n + 1) * 8));
        st.ins_ptr = dl.ins_ptr, st.del_ptr = dl.del_ptr, st.ent_ptr = dl.ent_ptr;
        ok = ok && st.cflags && st.cnt_ins && st.cnt_del && st.cnt_ent && st.row_flag && st.coffs && st.roffs && st.bits &&
             st.mask_del && st.mask_ins && st.mask_hit && dl.ins_ptr && dl.del_ptr && dl.ent_ptr;
        max_list = std::max(max_list, st.n_feat_rows);
        compare_features = compare_features || !b.feats_from_delta;
    }
    if (!ok) return nomem("scratch and row pointers");
    DiffStep *table_dev = static_cast<DiffStep *>(ctx->scratch(table.size() * sizeof(DiffStep)));
    if (!table_dev) return nomem("step table");
    const int sym = ctx->cfg.agg_kind == REINC_AGG_SYM;
    // job tables of the two scan stages and the table of totals, built up front and uploaded in one copy
    std::vector<ScanJob> jobs;
    jobs.reserve(size_t(5) * G);
    int64_t tiles[2] = {0, 0};
    auto add_job = [&](int stage, const int32_t *in, int64_t *out, int64_t count) {
        jobs.push_back(ScanJob{in, out, count, tiles[stage]});
        tiles[stage] += scan_tiles(count);
    };
    for (int g = 0; g < G; ++g) add_job(0, table[g].cflags, table[g].coffs, n);
    const int first_job1 = int(jobs.size());
    for (int g = 0; g < G; ++g) {
        add_job(1, table[g].cnt_ins, table[g].ins_ptr, n);
        add_job(1, table[g].cnt_del, table[g].del_ptr, n);
        add_job(1, table[g].cnt_ent, table[g].ent_ptr, n);
        add_job(1, table[g].row_flag, table[g].roffs, n);
    }
    constexpr int kTotals = 5;  // per step: inserted, deleted, entries, changed rows of S, changed nodes
    std::vector<const int64_t *> total_ptrs(size_t(kTotals) * G);
    for (int g = 0; g < G; ++g) {
        const DiffStep &st = table[g];
        const int64_t *p[kTotals] = {st.ins_ptr + n, st.del_ptr + n, st.ent_ptr + n, st.roffs + n, st.coffs + n};
        std::copy(p, p + kTotals, total_ptrs.begin() + size_t(kTotals) * g);
    }
    ScanJob *jobs_dev = static_cast<ScanJob *>(ctx->scratch(jobs.size() * sizeof(ScanJob)));
    const int64_t **ptrs_dev = static_cast<const int64_t **>(ctx->scratch(total_ptrs.size() * sizeof(int64_t *)));
    int64_t *totals_dev = i64s(int64_t(kTotals) * G);
    int64_t *tile_sums = i64s(std::max(tiles[0], tiles[1]));
    if (!jobs_dev || !ptrs_dev || !totals_dev || !tile_sums) return nomem("scan tables");
    REINC_HIP(ctx, hipMemcpyAsync(jobs_dev, jobs.data(), jobs.size() * sizeof(ScanJob), hipMemcpyHostToDevice, s));
    REINC_HIP(ctx, hipMemcpyAsync(ptrs_dev, total_ptrs.data(), total_ptrs.size() * sizeof(int64_t *), hipMemcpyHostToDevice, s));
    REINC_HIP(ctx, hipMemcpyAsync(table_dev, table.data(), table.size() * sizeof(DiffStep), hipMemcpyHostToDevice, s));
    auto stage = [&](int which, int64_t max_changed) {
        launch_diff_stage(which, table_dev, G, n, max_list, max_changed, sym, ctx->cfg.self_loop, bf16, d, s);
    };
    {
        ProfScope prof(ctx, REINC_K_DIFF, s);
        // stage 0: change sets C_t (steps whose features were loaded whole are compared row by row)
        stage(0, 0);
        if (compare_features)
            for (int g = 0; g < G; ++g) {
                const Snapshot &a = ctx->snaps[steps[g] - 1], &b = ctx->snaps[steps[g]];
                if (!b.feats_from_delta) launch_feature_flags_compare(a.x, b.x, n, d * ctx->elem_bytes(), table[g].cflags, s);
            }
        launch_multi_scan(jobs_dev, first_job1, tiles[0], tile_sums, s);
        // stage 1: per row, how many edges were inserted and deleted and how many entries the merged row gets; their
        // prefix sums over the rows are the row pointers of the outputs
        stage(1, 0);
        launch_multi_scan(jobs_dev + first_job1, int(jobs.size()) - first_job1, tiles[1], tile_sums, s);
    }
    launch_gather_i64(ptrs_dev, kTotals * G, totals_dev, s);
    std::vector<int64_t> totals(size_t(kTotals) * G);
    REINC_HIP(ctx, hipMemcpyAsync(totals.data(), totals_dev, totals.size() * 8, hipMemcpyDeviceToHost, s));
    REINC_HIP(ctx, hipStreamSynchronize(s));
    // stage 2: outputs of the sizes just learnt
    int64_t max_changed = 0;
    for (int g = 0; g < G; ++g) {
        const int64_t *tt = &totals[size_t(kTotals) * g];
        Delta &dl = ctx->deltas[steps[g]];
        auto take = [&](int64_t count, int64_t elem) { return ctx->alloc(uint64_t(std::max<int64_t>(count, 1)) * elem); };
        dl.changed = static_cast<int32_t *>(take(tt[4], 4));
        dl.dY = static_cast<float *>(take(tt[4], int64_t(d) * 4));
        dl.ins_col = static_cast<int32_t *>(take(tt[0], 4));
        dl.del_col = static_cast<int32_t *>(take(tt[1], 4));
        dl.ent = static_cast<uint32_t *>(take(tt[2], 4));
        dl.rows = static_cast<int32_t *>(take(tt[3], 4));
        dl.row_ent = static_cast<int64_t *>(take(tt[3] + 1, 8));
        if (!dl.changed || !dl.dY || !dl.ins_col || !dl.del_col || !dl.ent || !dl.rows || !dl.row_ent) return nomem("delta entries");
        DiffStep &st = table[g];
        st.ins_col = dl.ins_col, st.del_col = dl.del_col, st.ent = dl.ent;
        st.rows = dl.rows, st.row_ent = dl.row_ent, st.changed = dl.changed, st.dY = dl.dY;
        st.n_changed = tt[4];
        max_changed = std::max(max_changed, st.n_changed);
    }
    REINC_HIP(ctx, hipMemcpyAsync(table_dev, table.data(), table.size() * sizeof(DiffStep), hipMemcpyHostToDevice, s));
    {
        ProfScope prof(ctx, REINC_K_DIFF, s);
        stage(2, max_changed);
    }
    REINC_HIP(ctx, hipGetLastError());
    REINC_HIP(ctx, hipStreamSynchronize(s));
    ctx->scratch_reset();
    for (int g = 0; g < G; ++g) {
        const Snapshot &a = ctx->snaps[steps[g] - 1], &b = ctx->snaps[steps[g]];
        const int64_t *tt = &totals[size_t(kTotals) * g];
        Delta &dl = ctx->deltas[steps[g]];
        dl.info.num_edges_prev = a.nnz;
        dl.info.num_edges_cur = b.nnz;
        dl.info.n_ins = tt[0];
        dl.info.n_del = tt[1];
        dl.info.n_changed = tt[4];
        dl.info.n_entries = tt[2];
        dl.info.n_fchg_entries = tt[2] - tt[0] - tt[1];
        dl.info.n_rows = tt[3];
        dl.built = true;
    }
    return REINC_OK;
}

// Builds the given steps in groups as large as the free scratch allows (at least one step at a time).
static int build_steps(reinc_ctx *ctx, const std::vector<int32_t> &todo, hipStream_t s)
{
    const int64_t n = ctx->N();
    size_t i = 0;
    while (i < todo.size()) {
        ctx->scratch_reset();
        // room: what is free now, less the persistent outputs this group will take (row pointers now; entries bounded
        // by the edges of both snapshots, the changed rows and their features)
        const uint64_t room = ctx->top > ctx->bottom ? ctx->top - ctx->bottom : 0;
        uint64_t used = 0;
        std::vector<int32_t> group;
        while (i + group.size() < todo.size()) {
            const int32_t t = todo[i + group.size()];
            const Snapshot &a = ctx->snaps[t - 1], &b = ctx->snaps[t];
            const uint64_t persistent = 4 * uint64_t(n + 1) * 8 + uint64_t(2 * a.nnz + 3 * b.nnz + 4 * n) * 4 +
                                        uint64_t(n) * ctx->cfg.dims[0] * 4 + 16 * 256;
            const uint64_t tables = uint64_t(4 * n) / 256 + 4096;  // tile sums, job and pointer tables
            const uint64_t need = step_scratch_bytes(n, a.nnz, b.nnz) + persistent + tables;
            if (!group.empty() && used + need > room) break;
            used += need;
            group.push_back(t);
        }
        REINC_TRY(build_group(ctx, group, s));
        i += group.size();
    }
    return REINC_OK;
}

int reinc_build_deltas(reinc_ctx *ctx, int32_t t, void *stream)
{
    if (!ctx) return REINC_E_ARG;
    REINC_HIP(ctx, hipSetDevice(ctx->cfg.device));
    std::vector<int32_t> todo;
    if (t < 0) {
        for (int32_t k = 1; k < ctx->cfg.num_snapshots; ++k) {
            const Snapshot &a = ctx->snaps[k - 1], &b = ctx->snaps[k];
            if (a.edges_loaded && b.edges_loaded && a.feats_loaded && b.feats_loaded && !ctx->deltas[k].built) todo.push_back(k);
        }
        return build_steps(ctx, todo, as_stream(stream));
    }
    REINC_TRY(check_t(ctx, t));
    if (t == 0) return ctx->fail(REINC_E_ARG, "step 0 has no predecessor");
    if (ctx->deltas[t].built) return REINC_OK;
    const Snapshot &a = ctx->snaps[t - 1], &b = ctx->snaps[t];
    if (!a.edges_loaded || !b.edges_loaded || !a.feats_loaded || !b.feats_loaded)
        return ctx->fail(REINC_E_STATE, "step %d needs edges and features of snapshots %d and %d", t, t - 1, t);
    todo.push_back(t);
    return build_steps(ctx, todo, as_stream(stream));
}

static int need_delta(reinc_ctx *ctx, int32_t t)
{
    REINC_TRY(check_t(ctx, t));
    if (t == 0 || !ctx->deltas[t].built) return ctx->fail(REINC_E_STATE, "deltas of step %d are not built", t);
    return REINC_OK;
}

int reinc_get_delta_info(reinc_ctx *ctx, int32_t t, reinc_delta_info *out)
{
    if (!ctx || !out) return REINC_E_ARG;
    REINC_TRY(need_delta(ctx, t));
    *out = ctx->deltas[t].info;
    return REINC_OK;
}

int reinc_get_delta_csr(reinc_ctx *ctx, int32_t t, int kind, int64_t *row_ptr, int32_t *col, int64_t *nnz_out)
{
    if (!ctx) return REINC_E_ARG;
    REINC_TRY(need_delta(ctx, t));
    if (kind != 0 && kind != 1) return ctx->fail(REINC_E_ARG, "kind must be 0 (insert) or 1 (delete)");
    const Delta &dl = ctx->deltas[t];
    const int64_t nnz = kind == 0 ? dl.info.n_ins : dl.info.n_del;
    if (nnz_out) *nnz_out = nnz;
    REINC_TRY(read_back(ctx, row_ptr, kind == 0 ? dl.ins_ptr : dl.del_ptr, ctx->N() + 1));
    REINC_TRY(read_back(ctx, col, kind == 0 ? dl.ins_col : dl.del_col, nnz));
    return REINC_OK;
}

int reinc_get_merged_delta(reinc_ctx *ctx, int32_t t, int64_t *entry_ptr, uint32_t *entries, int32_t *rows,
                           int32_t *changed)
{
    if (!ctx) return REINC_E_ARG;
    REINC_TRY(need_delta(ctx, t));
    const Delta &dl = ctx->deltas[t];
    REINC_TRY(read_back(ctx, entry_ptr, dl.ent_ptr, ctx->N() + 1));
    REINC_TRY(read_back(ctx, entries, dl.ent, dl.info.n_entries));
    REINC_TRY(read_back(ctx, rows, dl.rows, dl.info.n_rows));
    REINC_TRY(read_back(ctx, changed, dl.changed, dl.info.n_changed));
    return REINC_OK;
}

int reinc_get_snapshot_csr(reinc_ctx *ctx, int32_t t, int transpose, int64_t *ptr, int32_t *idx, int64_t *nnz_out)
{
    if (!ctx) return REINC_E_ARG;
    REINC_TRY(check_t(ctx, t));
    const Snapshot &sn = ctx->snaps[t];
    if (!sn.edges_loaded) return ctx->fail(REINC_E_STATE, "edges of snapshot %d are not loaded", t);
    if (nnz_out) *nnz_out = sn.nnz;
    REINC_TRY(read_back(ctx, ptr, transpose ? sn.col_ptr : sn.row_ptr, ctx->N() + 1));
    REINC_TRY(read_back(ctx, idx, transpose ? sn.row : sn.col, sn.nnz));
    return REINC_OK;
}

// ------------------------------------------------------------------------------------------------ aggregation

int reinc_aggregate_full(reinc_ctx *ctx, int32_t t, int transpose, const void *X, int x_dtype, int32_t d, int apply_q,
                         float *out, void *stream)
{
    if (!ctx) return REINC_E_ARG;
    REINC_TRY(check_t(ctx, t));
    const Snapshot &sn = ctx->snaps[t];
    if (!sn.edges_loaded) return ctx->fail(REINC_E_STATE, "edges of snapshot %d are not loaded", t);
    if (!out) return ctx->fail(REINC_E_ARG, "null output");
    if (x_dtype != REINC_F32 && x_dtype != REINC_BF16) return ctx->fail(REINC_E_ARG, "bad x_dtype");
    if (!X) {
        if (!sn.feats_loaded) return ctx->fail(REINC_E_STATE, "features of snapshot %d are not loaded", t);
        if (d != ctx->cfg.dims[0] || x_dtype != ctx->cfg.feat_dtype)
            return ctx->fail(REINC_E_ARG, "stored features are [N, %d] of dtype %d", ctx->cfg.dims[0], ctx->cfg.feat_dtype);
        X = sn.x;
    }
    if (X == out) return ctx->fail(REINC_E_ARG, "output may not alias the input");
    if (!agg_width_supported(d, x_dtype == REINC_BF16))
        return ctx->fail(REINC_E_UNSUPPORTED, "row of %d elements: row bytes must be a power of two in [16, 1024]", d);
    const int bf16 = x_dtype == REINC_BF16;
    if (!transpose)
        aggregate_full(ctx, sn.row_ptr, sn.col, sn.long_rows, sn.n_long_rows, X, bf16, d, ctx->cfg.self_loop, sn.p,
                       apply_q ? sn.q : nullptr, nullptr, out, as_stream(stream), sn.row_order);
    else
        aggregate_full(ctx, sn.col_ptr, sn.row, sn.long_cols, sn.n_long_cols, X, bf16, d, ctx->cfg.self_loop,
                       apply_q ? sn.q : nullptr, sn.p, nullptr, out, as_stream(stream), sn.col_order);
    REINC_HIP(ctx, hipGetLastError());
    return REINC_OK;
}

int reinc_aggregate_incremental(reinc_ctx *ctx, int32_t t, const float *S_prev, float *S_out, float *agg_out,
                                void *stream)
{
    if (!ctx) return REINC_E_ARG;
    REINC_TRY(need_delta(ctx, t));
    if (!S_prev || !S_out) return ctx->fail(REINC_E_ARG, "null aggregate buffer");
    const Delta &dl = ctx->deltas[t];
    const Snapshot &pv = ctx->snaps[t - 1];
    const Snapshot &sn = ctx->snaps[t];
    const int32_t d = ctx->cfg.dims[0];
    const uint64_t bytes = uint64_t(ctx->N()) * d * 4;
    const bool in_place = S_out == S_prev;
    if (!in_place) {
        const char *a = reinterpret_cast<const char *>(S_prev), *b = reinterpret_cast<const char *>(S_out);
        if (a < b + bytes && b < a + bytes) return ctx->fail(REINC_E_ARG, "S_out must be S_prev itself or disjoint from it");
        if (agg_out) return ctx->fail(REINC_E_ARG, "agg_out is only updated in place: pass S_out == S_prev with it");
    }
    {
        // in place: the rows of R_t; to a new buffer: one pass over every row (rows without entries are copied)
        ProfScope prof(ctx, REINC_K_AGG_INC, as_stream(stream), true);
        launch_incremental(in_place ? dl.rows : nullptr, dl.row_ent, in_place ? dl.info.n_rows : ctx->N(), dl.ent_ptr, dl.ent, pv.x,
                           ctx->cfg.feat_dtype == REINC_BF16, pv.p, dl.dY, d, S_prev, S_out, sn.q, agg_out, as_stream(stream),
                           prof.start(), prof.stop());
    }
    REINC_HIP(ctx, hipGetLastError());
    ctx->stats.delta_entries_processed += dl.info.n_entries;
    return REINC_OK;
}

int reinc_aggregate_full_minmax(reinc_ctx *ctx, int32_t t, int op, const void *X, int x_dtype, int32_t d, float *out,
                                int32_t *contrib, void *stream)
{
    if (!ctx) return REINC_E_ARG;
    REINC_TRY(check_t(ctx, t));
    const Snapshot &sn = ctx->snaps[t];
    if (!sn.edges_loaded) return ctx->fail(REINC_E_STATE, "edges of snapshot %d are not loaded", t);
    if (op != REINC_OP_MAX && op != REINC_OP_MIN) return ctx->fail(REINC_E_ARG, "op must be REINC_OP_MAX or REINC_OP_MIN");
    if (!out || !contrib) return ctx->fail(REINC_E_ARG, "null output");
    if (x_dtype != REINC_F32 && x_dtype != REINC_BF16) return ctx->fail(REINC_E_ARG, "bad x_dtype");
    if (!X) {
        if (!sn.feats_loaded) return ctx->fail(REINC_E_STATE, "features of snapshot %d are not loaded", t);
        if (d != ctx->cfg.dims[0] || x_dtype != ctx->cfg.feat_dtype)
            return ctx->fail(REINC_E_ARG, "stored features are [N, %d] of dtype %d", ctx->cfg.dims[0], ctx->cfg.feat_dtype);
        X = sn.x;
    }
    if (X == out) return ctx->fail(REINC_E_ARG, "output may not alias the input");
    if (!agg_width_supported(d, x_dtype == REINC_BF16))
        return ctx->fail(REINC_E_UNSUPPORTED, "row of %d elements: row bytes must be a power of two in [16, 1024]", d);
    {
        ProfScope prof(ctx, REINC_K_AGG_MINMAX, as_stream(stream));
        launch_minmax_full(sn.row_ptr, sn.col, sn.long_rows, sn.n_long_rows, X, x_dtype == REINC_BF16, d, ctx->N(),
                           ctx->cfg.self_loop, op == REINC_OP_MAX, out, contrib, as_stream(stream));
    }
    REINC_HIP(ctx, hipGetLastError());
    return REINC_OK;
}

int reinc_aggregate_incremental_minmax(reinc_ctx *ctx, int32_t t, int op, const float *M_prev, const int32_t *C_prev,
                                       float *M_out, int32_t *C_out, int32_t *work, void *stream)
{
    if (!ctx) return REINC_E_ARG;
    return reinc::minmax_incremental(ctx, t, op, M_prev, C_prev, M_out, C_out, work, true, as_stream(stream));
}

extern "C++" int reinc::minmax_incremental(reinc_ctx *ctx, int32_t t, int op, const float *M_prev, const int32_t *C_prev,
                                           float *M_out, int32_t *C_out, int32_t *work, bool timed, hipStream_t s)
{
    REINC_TRY(need_delta(ctx, t));
    if (op != REINC_OP_MAX && op != REINC_OP_MIN) return ctx->fail(REINC_E_ARG, "op must be REINC_OP_MAX or REINC_OP_MIN");
    if (!M_prev || !C_prev || !M_out || !C_out || !work) return ctx->fail(REINC_E_ARG, "null buffer");
    const Delta &dl = ctx->deltas[t];
    const Snapshot &sn = ctx->snaps[t];
    const int32_t d = ctx->cfg.dims[0];
    const uint64_t bytes = uint64_t(ctx->N()) * d * 4;
    const bool in_place = M_out == M_prev;
    if (in_place != (C_out == C_prev))
        return ctx->fail(REINC_E_ARG, "values and contributors must both be updated in place or both go to new buffers");
    if (!in_place) {
        const char *a = reinterpret_cast<const char *>(M_prev), *b = reinterpret_cast<const char *>(M_out);
        const char *e = reinterpret_cast<const char *>(C_prev), *f = reinterpret_cast<const char *>(C_out);
        if ((a < b + bytes && b < a + bytes) || (e < f + bytes && f < e + bytes))
            return ctx->fail(REINC_E_ARG, "output buffers must be the previous ones themselves or disjoint from them");
    }
    // work: [0] rows aggregated from scratch, [1] spare, [2, N+2) hub-row marks by row id, then per-block counts.
    // Everything that must start at zero is cleared here, by a kernel: the buffer keeps the last call's contents.
    launch_fill_f32(reinterpret_cast<float *>(work), ctx->N() + 2, 0.0f, s);  // (bit pattern 0)
    {
        const int64_t n_rows = in_place ? dl.info.n_rows : ctx->N();
        auto run = [&] {
            launch_minmax_incremental(in_place ? dl.rows : nullptr, n_rows, sn.long_rows, sn.n_long_rows, dl.ent_ptr, dl.ent,
                                      dl.changed, sn.row_ptr, sn.col, sn.x, ctx->cfg.feat_dtype == REINC_BF16, d,
                                      ctx->cfg.self_loop, op == REINC_OP_MAX, M_prev, C_prev, M_out, C_out, work + 2,
                                      work + 2 + ctx->N(), work, s);
        };
        if (timed) {
            ProfScope prof(ctx, REINC_K_AGG_MINMAX, s);  // (creates events while a profile is open)
            run();
        } else {
            run();
        }
    }
    REINC_HIP(ctx, hipGetLastError());
    return REINC_OK;
}

int reinc_reset_derived(reinc_ctx *ctx)
{
    if (!ctx) return REINC_E_ARG;
    if (!ctx->has_derived) return REINC_OK;
    if (ctx->load_after_derived)
        return ctx->fail(REINC_E_STATE, "a snapshot was loaded after deltas or caches were built: their space cannot be returned");
    REINC_HIP(ctx, hipSetDevice(ctx->cfg.device));
    REINC_HIP(ctx, hipDeviceSynchronize());
    ctx->bottom = ctx->derived_mark;
    ctx->has_derived = false;
    for (Delta &d : ctx->deltas) d = Delta();
    std::fill(ctx->gcache.begin(), ctx->gcache.end(), nullptr);
    // the cache buffers went back to the arena with everything else; a configured budget stays in force
    ctx->pool.clear();
    ctx->pool_free.clear();
    ctx->pending.clear();
    ctx->expired_pending.clear();
    if (ctx->gpolicy) ctx->gpolicy->clear();
    ctx->local.clear();
    ctx->local_L = 0;
    ctx->local_kind = 0;
    ctx->local_valid = false;
    ctx->local_reserved = 0;
    ctx->zero_state = nullptr;
    ctx->loss_partial = nullptr;
    ctx->batch_level = ctx->batch_new_id = ctx->batch_nodes = nullptr;  // a mini-batch plan lived above the mark
    ctx->batch_total = ctx->batch_size = 0;
    ctx->stats.local_bytes = 0;
    ctx->scratch_reset();
    return REINC_OK;
}

int reinc_sgd_step(reinc_ctx *ctx, float *params, const float *grads, int64_t count, float lr, void *stream)
{
    if (!ctx) return REINC_E_ARG;
    if (!params || !grads || count < 0) return ctx->fail(REINC_E_ARG, "null params or grads");
    launch_sgd(params, grads, count, lr, as_stream(stream));
    REINC_HIP(ctx, hipGetLastError());
    return REINC_OK;
}

int reinc_profile_begin(reinc_ctx *ctx, uint32_t mask)
{
    if (!ctx) return REINC_E_ARG;
    ctx->prof_kind.clear();
    ctx->prof_mask = mask;
    return REINC_OK;
}

int reinc_profile_end(reinc_ctx *ctx, int64_t *launches, double *total_ms)
{
    if (!ctx || !launches || !total_ms) return REINC_E_ARG;
    ctx->prof_mask = 0;
    REINC_HIP(ctx, hipSetDevice(ctx->cfg.device));
    REINC_HIP(ctx, hipDeviceSynchronize());
    for (int k = 0; k < REINC_K_COUNT; ++k) {
        launches[k] = 0;
        total_ms[k] = 0.0;
    }
    for (size_t i = 0; i < ctx->prof_kind.size(); ++i) {
        float ms = 0.0f;
        REINC_HIP(ctx, hipEventElapsedTime(&ms, ctx->prof_events[2 * i], ctx->prof_events[2 * i + 1]));
        launches[ctx->prof_kind[i]] += 1;
        total_ms[ctx->prof_kind[i]] += double(ms);
    }
    ctx->prof_kind.clear();
    return REINC_OK;
}

int reinc_get_stats(reinc_ctx *ctx, reinc_stats *out)
{
    if (!ctx || !out) return REINC_E_ARG;
    ctx->stats.arena_used = int64_t(ctx->bottom);
    ctx->stats.arena_peak = int64_t(ctx->peak);
    ctx->sync_policy_stats();
    *out = ctx->stats;
    return REINC_OK;
}

}  // extern "C"
