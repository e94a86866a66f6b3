// Dense-step entry points and the window driver with its two caches (paper Section 2.2: a window of L
// consecutive snapshots is one training sample with back-propagation through time; Section 3.3: a global
// cache for the aggregates of the input features, a local cache for per-layer intermediates).
#include <algorithm>
#include <initializer_list>
#include <vector>

#include "ctx.h"

#include <new>

using namespace reinc;

namespace {

hipStream_t as_stream(void *s) { return static_cast<hipStream_t>(s); }

// launch wrappers that time the kernel class when profiling is on
template <class... A>
void gemm_rows(reinc_ctx *ctx, hipStream_t st, A... a)
{
    ProfScope prof(ctx, REINC_K_GEMM_ROWS, st);
    launch_gemm_rows(a..., st);
}
template <class... A>
void rnn_fused(reinc_ctx *ctx, hipStream_t st, A... a)
{
    ProfScope prof(ctx, REINC_K_RNN, st);
    launch_rnn_fused(a..., st);
}
template <class... A>
void gemm_reduce(reinc_ctx *ctx, hipStream_t st, A... a)
{
    ProfScope prof(ctx, REINC_K_REDUCE, st);
    launch_gemm_reduce(a..., st);
}
template <class... A>
void rnn_backward_elem(reinc_ctx *ctx, hipStream_t st, A... a)
{
    ProfScope prof(ctx, REINC_K_ELEM, st);
    launch_rnn_backward_elem(a..., st);
}

struct Params {
    const float *W[REINC_MAX_GCN_LAYERS + 1] = {};
    const float *b[REINC_MAX_GCN_LAYERS + 1] = {};
    const float *W_i = nullptr, *W_h = nullptr, *b_i = nullptr, *b_h = nullptr;
    int64_t count = 0;
};

// flat layout: per layer W_l [d_{l-1}, d_l], b_l [d_l]; then W_i [d_last, K*H], W_h [H, K*H], b_i, b_h
Params split_params(const reinc_config &c, const float *flat)
{
    Params p;
    int64_t off = 0;
    for (int l = 1; l <= c.num_gcn_layers; ++l) {
        p.W[l] = flat + off;
        off += int64_t(c.dims[l - 1]) * c.dims[l];
        p.b[l] = flat + off;
        off += c.dims[l];
    }
    const int64_t kh = int64_t(c.rnn_kind == REINC_RNN_LSTM ? 4 : 3) * c.rnn_hidden;
    p.W_i = flat + off;
    off += int64_t(c.dims[c.num_gcn_layers]) * kh;
    p.W_h = flat + off;
    off += int64_t(c.rnn_hidden) * kh;
    p.b_i = flat + off;
    off += kh;
    p.b_h = flat + off;
    off += kh;
    p.count = off;
    return p;
}

uint64_t align256(uint64_t b) { return (b + 255) & ~uint64_t(255); }

// Layers above the first whose output is narrower than their input apply the linear map BEFORE the aggregation:
// A (H W) = (A H) W, the same layer within rounding, but every edge then gathers a row of dims[l] values instead of
// dims[l-1] (the gathers of these layers are the largest share of a step when the widths shrink).  Z = H W stays in
// fp32: kept in bfloat16 (tried for bfloat16 node features) it halves the gathered bytes again, but the rounding moves
// enough ReLU decisions of the layer that single weight-gradient entries of a 1200-node graph miss the 2e-2 bound.
bool transform_first(const reinc_config &c, int l) { return l >= 2 && c.dims[l] < c.dims[l - 1]; }
// floats a timestep's rows of LocalStep::S[l] take: the sums feeding layer l, or Z of a transform-first layer
uint64_t s_width_floats(const reinc_config &c, int l) { return uint64_t(transform_first(c, l) ? c.dims[l] : c.dims[l - 1]); }

// The local cache keeps every quantity as one array over the window's timesteps, so that the rows of consecutive
// timesteps are adjacent and the dense kernels can take a whole batch of timesteps as one tall matrix.  A
// timestep's slice is exactly n*d floats when that keeps slices 16-byte aligned, else it is padded (and the
// driver falls back to one launch per timestep for that quantity).
uint64_t slice_floats(uint64_t n, uint64_t d) { return (n * d) % 4 == 0 ? n * d : align256(n * d * 4) / 4; }

uint64_t local_bytes(const reinc_config &c, int32_t L)
{
    const uint64_t n = uint64_t(c.num_nodes), H = uint64_t(c.rnn_hidden);
    uint64_t b = 0;
    for (int l = 1; l <= c.num_gcn_layers; ++l) {
        b += align256(uint64_t(L) * slice_floats(n, c.dims[l]) * 4);
        if (l >= 2) b += align256(uint64_t(L) * slice_floats(n, s_width_floats(c, l)) * 4);
    }
    b += align256(uint64_t(L + 1) * slice_floats(n, H) * 4);                                  // h, with the zero state in front
    if (c.rnn_kind == REINC_RNN_LSTM) b += align256(uint64_t(L) * slice_floats(n, H) * 4);    // c
    b += align256(uint64_t(L) * slice_floats(n, 4 * H) * 4);                                  // gate values
    return b;
}

// The local cache holds the last `local_reserved` bytes of the arena; it is re-carved when a longer window arrives.
int ensure_local(reinc_ctx *ctx, int32_t L, hipStream_t s)
{
    const reinc_config &c = ctx->cfg;
    if (ctx->local_kind == 0 && ctx->local_L >= L && !ctx->local.empty()) return REINC_OK;
    const uint64_t n = uint64_t(c.num_nodes), H = uint64_t(c.rnn_hidden);
    const uint64_t need = align256(loss_partial_bytes()) + local_bytes(c, L);
    if (ctx->bottom + need > ctx->size)
        return ctx->fail(REINC_E_NOMEM, "arena exhausted: the local cache of a %d-step window needs %llu bytes", L,
                         (unsigned long long)need);
    ctx->local_reserved = need;
    ctx->scratch_reset();
    char *p = ctx->base + (ctx->size - need);
    auto take = [&](uint64_t bytes) {
        char *r = p;
        p += align256(bytes);
        return reinterpret_cast<float *>(r);
    };
    ctx->loss_partial = take(loss_partial_bytes());
    ctx->local.assign(L, LocalStep());
    for (int l = 1; l <= c.num_gcn_layers; ++l) {
        const uint64_t sh = slice_floats(n, c.dims[l]);
        float *Hl = take(uint64_t(L) * sh * 4);
        for (int32_t i = 0; i < L; ++i) ctx->local[i].H[l] = Hl + i * sh;
        if (l >= 2) {
            const uint64_t ss = slice_floats(n, s_width_floats(c, l));
            float *Sl = take(uint64_t(L) * ss * 4);
            for (int32_t i = 0; i < L; ++i) ctx->local[i].S[l] = Sl + i * ss;
        }
    }
    {
        const uint64_t sh = slice_floats(n, H);
        float *h = take(uint64_t(L + 1) * sh * 4);
        ctx->zero_state = h;  // the state before timestep 0: h_{t-1} of timestep i is slice i
        for (int32_t i = 0; i < L; ++i) ctx->local[i].h = h + (i + 1) * sh;
        if (c.rnn_kind == REINC_RNN_LSTM) {
            float *cs = take(uint64_t(L) * sh * 4);
            for (int32_t i = 0; i < L; ++i) ctx->local[i].c = cs + i * sh;
        }
        const uint64_t sg = slice_floats(n, 4 * H);
        float *sv = take(uint64_t(L) * sg * 4);
        for (int32_t i = 0; i < L; ++i) ctx->local[i].saved = sv + i * sg;
    }
    ctx->local_L = L;
    ctx->local_kind = 0;
    ctx->local_valid = false;
    ctx->local_top = int64_t(n);
    ctx->stats.local_bytes = int64_t(need);
    launch_fill_f32(ctx->zero_state, int64_t(n) * c.rnn_hidden, 0.0f, s);
    return REINC_OK;
}

// Not every layer is computed on every row: with loss rows set (a node mini-batch, numbered first) the last GCN layer
// and the recurrent cell work on those `nt` rows only, and a batch context may know that a layer below is needed on
// its first rows only (reinc_ctx::rows_of_layer).  The per-timestep slices of a quantity are placed as many rows apart
// as it has, inside the allocations ensure_local made for N rows, so that consecutive timesteps stay adjacent rows of
// one tall matrix.  Z = H W of a layer that narrows its input has the rows of the layer below (they are sources).
void place_rows(reinc_ctx *ctx, hipStream_t s)
{
    const reinc_config &c = ctx->cfg;
    const int Lg = c.num_gcn_layers;
    const int64_t nt = ctx->top_rows();
    const uint64_t H = uint64_t(c.rnn_hidden), rows = uint64_t(nt);
    float *bH[REINC_MAX_GCN_LAYERS + 1] = {}, *bS[REINC_MAX_GCN_LAYERS + 1] = {};
    for (int l = 1; l <= Lg; ++l) {
        bH[l] = ctx->local[0].H[l];
        bS[l] = l >= 2 ? ctx->local[0].S[l] : nullptr;
        ctx->local_rows[l] = ctx->rows_of_layer(l);
    }
    float *bc = ctx->local[0].c, *bsv = ctx->local[0].saved;
    for (size_t i = 0; i < ctx->local.size(); ++i) {
        reinc::LocalStep &st = ctx->local[i];
        for (int l = 1; l <= Lg; ++l) {
            const uint64_t rl = uint64_t(ctx->rows_of_layer(l));
            st.H[l] = bH[l] + i * slice_floats(rl, c.dims[l]);
            if (l >= 2) st.S[l] = bS[l] + i * slice_floats(transform_first(c, l) ? uint64_t(ctx->rows_of_layer(l - 1)) : rl, s_width_floats(c, l));
        }
        st.h = ctx->zero_state + (i + 1) * slice_floats(rows, H);
        if (bc) st.c = bc + i * slice_floats(rows, H);
        st.saved = bsv + i * slice_floats(rows, 4 * H);
    }
    if (ctx->local_top != nt) {  // another placement wrote states where the zero state of this one lies
        launch_fill_f32(ctx->zero_state, nt * c.rnn_hidden, 0.0f, s);
        ctx->local_top = nt;
    }
}

// dst[i * rows + r] = src_i[r] for the timesteps i of a batch: the degree scales of a layer that works on its first
// rows only, next to each other like the layer's other per-timestep quantities
struct ScaleTable {
    const float *src[kMaxAggBatch];
};
__global__ void gather_scales(ScaleTable t, int64_t rows, float *dst)
{
    const int64_t r = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (r < rows) dst[int64_t(blockIdx.y) * rows + r] = t.src[blockIdx.y][r];
}

// Local cache of the integrated model: per timestep the aggregated hidden state Agg(h_{t-1}) (kept in LocalStep::S[1];
// slice 0 stays zero: the state before the window is zero), the state h (zero state in front), c, the gate values.
int ensure_local_integrated(reinc_ctx *ctx, int32_t L, hipStream_t s)
{
    const reinc_config &c = ctx->cfg;
    if (ctx->local_kind == 1 && ctx->local_L >= L && !ctx->local.empty()) return REINC_OK;
    const uint64_t n = uint64_t(c.num_nodes), H = uint64_t(c.rnn_hidden);
    const uint64_t sh = slice_floats(n, H), sg = slice_floats(n, 4 * H);
    const bool lstm = c.rnn_kind == REINC_RNN_LSTM;
    const uint64_t need = align256(loss_partial_bytes()) + align256(uint64_t(L) * sh * 4) + align256(uint64_t(L + 1) * sh * 4) +
                          (lstm ? align256(uint64_t(L) * sh * 4) : 0) + align256(uint64_t(L) * sg * 4);
    if (ctx->bottom + need > ctx->size)
        return ctx->fail(REINC_E_NOMEM, "arena exhausted: the local cache of a %d-step window needs %llu bytes", L,
                         (unsigned long long)need);
    ctx->local_reserved = need;
    ctx->scratch_reset();
    char *p = ctx->base + (ctx->size - need);
    auto take = [&](uint64_t bytes) {
        char *r = p;
        p += align256(bytes);
        return reinterpret_cast<float *>(r);
    };
    ctx->loss_partial = take(loss_partial_bytes());
    ctx->local.assign(L, LocalStep());
    float *ah = take(uint64_t(L) * sh * 4), *h = take(uint64_t(L + 1) * sh * 4);
    float *cs = lstm ? take(uint64_t(L) * sh * 4) : nullptr;
    float *sv = take(uint64_t(L) * sg * 4);
    ctx->zero_state = h;
    for (int32_t i = 0; i < L; ++i) {
        ctx->local[i].S[1] = ah + i * sh;
        ctx->local[i].h = h + (i + 1) * sh;
        ctx->local[i].c = cs ? cs + i * sh : nullptr;
        ctx->local[i].saved = sv + i * sg;
    }
    ctx->local_L = L;
    ctx->local_kind = 1;
    ctx->local_valid = false;
    ctx->stats.local_bytes = int64_t(need);
    launch_fill_f32(ctx->zero_state, int64_t(n) * c.rnn_hidden, 0.0f, s);
    launch_fill_f32(ah, int64_t(n) * c.rnn_hidden, 0.0f, s);
    return REINC_OK;
}

uint64_t aggregate_bytes(const reinc_config &c) { return align256(uint64_t(c.num_nodes) * c.dims[0] * 4); }

// Budgeted cache: takes the buffers (what may be retained plus one window's worth) from the arena, once.
int ensure_pool(reinc_ctx *ctx)
{
    const uint64_t want = uint64_t(ctx->budget_slots) + uint64_t(ctx->plan_window);
    if (ctx->pool.size() >= want) return REINC_OK;
    const uint64_t bytes = aggregate_bytes(ctx->cfg);
    ctx->note_derived();
    while (ctx->pool.size() < want) {
        float *b = static_cast<float *>(ctx->alloc(bytes));
        if (!b)
            return ctx->fail(REINC_E_NOMEM, "arena exhausted: the cache budget needs %llu buffers of %llu bytes",
                             (unsigned long long)want, (unsigned long long)bytes);
        ctx->pool.push_back(b);
        ctx->pool_free.push_back(b);
    }
    return REINC_OK;
}

// Budgeted cache: the previous window is over.  Buffers of its expired hits return to the pool, and what it computed
// is offered to the policy in snapshot order (Section 3.3, eviction policy: F / S - I with expiration, or LRU / LFU).
void retire_window(reinc_ctx *ctx)
{
    if (!ctx->gpolicy) return;
    auto release = [&](int32_t t) {
        if (ctx->gcache[t]) ctx->pool_free.push_back(ctx->gcache[t]);
        ctx->gcache[t] = nullptr;
    };
    for (int32_t t : ctx->expired_pending) release(t);
    ctx->expired_pending.clear();
    const int64_t T = ctx->cfg.num_snapshots, S = ctx->plan_stride, t0 = ctx->pending_t0, L = ctx->pending_L;
    const int64_t size = int64_t(aggregate_bytes(ctx->cfg));
    std::vector<int64_t> gone;
    for (int32_t t : ctx->pending) {
        // later windows of the epoch (starts t0 + S, t0 + 2S, ... up to T - L) that still contain snapshot t
        const int64_t future = std::max<int64_t>(std::min((t - t0) / S, (T - L - t0) / S), 0);
        gone.clear();
        const bool kept = ctx->gpolicy->offer(t, size, future, L - S, &gone);
        for (int64_t k : gone) release(int32_t(k));
        if (!kept) release(t);
    }
    ctx->pending.clear();
    ctx->sync_policy_stats();
}

// Budgeted cache, start of a forward window: settle the previous window, then note the new one.
int begin_budgeted_window(reinc_ctx *ctx, int32_t t0, int32_t L)
{
    if (!ctx->gpolicy) return REINC_OK;
    if (L > ctx->plan_window)
        return ctx->fail(REINC_E_ARG, "window of %d steps, but the cache budget was configured for at most %d", L, ctx->plan_window);
    ctx->scratch_reset();  // scratch of the previous call is dead: the buffers may use that room
    REINC_TRY(ensure_pool(ctx));
    retire_window(ctx);
    ctx->pending_t0 = t0;
    ctx->pending_L = L;
    return REINC_OK;
}

// Makes sure the layer-1 sums of snapshot t are available: ctx->gcache[t] points at them afterwards.
int ensure_layer1(reinc_ctx *ctx, int32_t t, hipStream_t s)
{
    const reinc_config &c = ctx->cfg;
    if (ctx->gpolicy) {
        bool expired = false;
        if (ctx->gpolicy->access(t, &expired)) {
            ++ctx->stats.global_hits;
            if (expired) ctx->expired_pending.push_back(t);  // the buffer stays ours until this window is retired
            return REINC_OK;
        }
    } else if (ctx->gcache[t]) {
        ++ctx->stats.global_hits;
        return REINC_OK;
    }
    const Snapshot &sn = ctx->snaps[t];
    if (!sn.edges_loaded || !sn.feats_loaded)
        return ctx->fail(REINC_E_STATE, "snapshot %d needs its edges and features loaded", t);
    const int32_t d = c.dims[0];
    const int bf16 = c.feat_dtype == REINC_BF16;
    const int64_t rows = ctx->cached_rows();  // (a batch context: the rows layer 1 is needed on; the buffer is that short)
    const uint64_t bytes = uint64_t(rows) * d * 4;
    float *slot = nullptr;
    if (ctx->gpolicy) {
        if (ctx->pool_free.empty()) return ctx->fail(REINC_E_STATE, "cache buffers exhausted (window longer than configured?)");
        // the dense kernels take consecutive timesteps as one tall matrix when their sums are adjacent in memory:
        // prefer the buffer right behind the previous snapshot's, else the lowest free address (the retained
        // window then moves through the pool like a ring)
        auto pick = std::min_element(ctx->pool_free.begin(), ctx->pool_free.end());
        if (t > 0 && ctx->gcache[t - 1]) {
            float *next = reinterpret_cast<float *>(reinterpret_cast<char *>(ctx->gcache[t - 1]) + aggregate_bytes(c));
            auto it = std::find(ctx->pool_free.begin(), ctx->pool_free.end(), next);
            if (it != ctx->pool_free.end()) pick = it;
        }
        slot = *pick;
        ctx->pool_free.erase(pick);
        ctx->gcache[t] = slot;  // recorded before anything can fail, so that the buffer always finds its way back
        ctx->pending.push_back(t);
    } else {
        ctx->note_derived();
        slot = static_cast<float *>(ctx->alloc(bytes));
        if (!slot) return ctx->fail(REINC_E_NOMEM, "arena exhausted: no room for the cached aggregate of snapshot %d", t);
    }
    ++ctx->stats.global_misses;
    const bool chain = t > 0 && ctx->gcache[t - 1] && ctx->deltas[t].built && c.fallback_ratio != 0.0f;
    bool incremental = chain;
    if (chain && c.fallback_ratio > 0.0f) {
        const reinc_delta_info &di = ctx->deltas[t].info;
        const double ratio = double(di.n_entries) / double(std::max<int64_t>(di.num_edges_cur, 1));
        if (ratio > double(c.fallback_ratio)) {
            incremental = false;
            ++ctx->stats.steps_fallback;
        }
    }
    if (incremental) {
        const Delta &dl = ctx->deltas[t];
        const Snapshot &pv = ctx->snaps[t - 1];
        {
            // one pass over every row: changed rows get their delta, the others are copied into the new slot
            ProfScope prof(ctx, REINC_K_AGG_INC, s, true);
            launch_incremental(nullptr, nullptr, rows, dl.ent_ptr, dl.ent, pv.x, bf16, pv.p, dl.dY, d, ctx->gcache[t - 1], slot,
                               nullptr, nullptr, s, prof.start(), prof.stop());
        }
        ++ctx->stats.steps_incremental;
        ctx->stats.delta_entries_processed += dl.info.n_entries;
    } else {
        AggBatch batch;
        batch.count = 1;
        batch.item[0] = AggItem{sn.row_ptr, sn.col, sn.x, sn.p, nullptr, nullptr, nullptr, slot, sn.long_rows, sn.n_long_rows};
        if (rows < c.num_nodes)
            batch.item[0].row_limit = rows;
        else
            batch.item[0].order = sn.row_order;
        aggregate_full_batch(ctx, batch, bf16, d, c.self_loop, s, rows);
        ++ctx->stats.steps_full;
    }
    REINC_HIP(ctx, hipGetLastError());
    ctx->gcache[t] = slot;
    return REINC_OK;
}

int check_window(reinc_ctx *ctx, int32_t t0, int32_t L)
{
    if (t0 < 0 || L < 1 || int64_t(t0) + L > ctx->cfg.num_snapshots)
        return ctx->fail(REINC_E_ARG, "window [%d, %d) outside [0, %d)", t0, t0 + L, ctx->cfg.num_snapshots);
    return REINC_OK;
}

// Calls fn(i0, len) for every maximal run of timesteps [i0, i0 + len) of [lo, hi] whose rows are adjacent in memory in
// each of the given per-timestep arrays: such a run is one tall matrix of n * len rows.
struct Strip {
    const float *const *each;  // start of every timestep's [n, row_floats] array, indexed by timestep; null: ignore
    int64_t row_floats;
};

template <class F>
int for_runs(int lo, int hi, int64_t n, std::initializer_list<Strip> strips, F fn)
{
    int i0 = lo;
    while (i0 <= hi) {
        int len = 1;
        for (; i0 + len <= hi; ++len) {
            bool adjacent = true;
            for (const Strip &st : strips)
                if (st.each && st.each[i0 + len] != st.each[i0 + len - 1] + n * st.row_floats) adjacent = false;
            if (!adjacent) break;
        }
        const int rc = fn(i0, len);
        if (rc != REINC_OK) return rc;
        i0 += len;
    }
    return REINC_OK;
}

}  // namespace

extern "C" {

int reinc_gcn_transform(reinc_ctx *ctx, const void *A, int a_dtype, int64_t n, int32_t d_in, int32_t d_out,
                        const float *row_scale, const float *W, const float *b, int relu, float *out, void *stream)
{
    if (!ctx) return REINC_E_ARG;
    if (!A || !W || !out) return ctx->fail(REINC_E_ARG, "null matrix");
    if (n < 0 || d_in <= 0 || d_out <= 0) return ctx->fail(REINC_E_ARG, "bad shape");
    if (a_dtype != REINC_F32 && a_dtype != REINC_BF16) return ctx->fail(REINC_E_ARG, "bad a_dtype");
    if (A == out) return ctx->fail(REINC_E_ARG, "output may not alias the input");
    gemm_rows(ctx, as_stream(stream), A, int(a_dtype == REINC_BF16), n, d_in, d_out, row_scale, W, 0, d_out, b, relu,
              (const float *)nullptr, (const float *)nullptr, out);
    REINC_HIP(ctx, hipGetLastError());
    return REINC_OK;
}

int reinc_rnn_step(reinc_ctx *ctx, int rnn_kind, const float *x, int64_t n, int32_t d_in, int32_t H, const float *h_prev,
                   const float *c_prev, const float *W_i, const float *W_h, const float *b_i, const float *b_h,
                   float *h_out, float *c_out, float *saved, void *stream)
{
    if (!ctx) return REINC_E_ARG;
    if (rnn_kind != REINC_RNN_GRU && rnn_kind != REINC_RNN_LSTM) return ctx->fail(REINC_E_ARG, "bad rnn_kind");
    if (!x || !W_i || !W_h || !h_out) return ctx->fail(REINC_E_ARG, "null matrix");
    if (rnn_kind == REINC_RNN_LSTM && !c_out) return ctx->fail(REINC_E_ARG, "an LSTM step needs c_out");
    if (n < 0 || d_in <= 0 || H <= 0) return ctx->fail(REINC_E_ARG, "bad shape");
    if (h_out == h_prev || (c_out && c_out == c_prev)) return ctx->fail(REINC_E_ARG, "state outputs may not alias the previous state");
    rnn_fused(ctx, as_stream(stream), int(rnn_kind == REINC_RNN_LSTM), x, static_cast<const float *>(nullptr), n, d_in, H, h_prev,
              h_prev, c_prev, W_i, W_h, b_i, b_h, h_out, c_out, saved);
    REINC_HIP(ctx, hipGetLastError());
    return REINC_OK;
}

int reinc_forward_window(reinc_ctx *ctx, int32_t t0, int32_t L, const float *params, const float *target, float *loss_out,
                         float *h_last, void *stream)
{
    if (!ctx) return REINC_E_ARG;
    REINC_TRY(check_window(ctx, t0, L));
    if (!params) return ctx->fail(REINC_E_ARG, "null parameter vector");
    if (target && !loss_out) return ctx->fail(REINC_E_ARG, "a target needs loss_out");
    const reinc_config &c = ctx->cfg;
    for (int l = 2; l <= c.num_gcn_layers; ++l) {  // what layer l aggregates: its input rows, or Z = H W of its own width
        const bool tf = transform_first(c, l);
        if (!agg_width_supported(tf ? c.dims[l] : c.dims[l - 1], 0))
            return ctx->fail(REINC_E_UNSUPPORTED, "layer %d aggregates rows of %d values: row bytes must be a power of two in [16, 1024]",
                             l, tf ? c.dims[l] : c.dims[l - 1]);
    }
    hipStream_t s = as_stream(stream);
    REINC_HIP(ctx, hipSetDevice(c.device));
    ctx->local_valid = false;
    if (ctx->cache_rows > 0 && ctx->cache_rows < ctx->rows_of_layer(1)) {
        // (a batch context whose cached sums were made for a short window of the integrated model: too few rows)
        REINC_TRY(reinc_cache_clear(ctx));
        ctx->cache_rows = ctx->rows_of_layer(1) < c.num_nodes ? ctx->rows_of_layer(1) : 0;
    }
    REINC_TRY(begin_budgeted_window(ctx, t0, L));
    REINC_TRY(ensure_local(ctx, L, s));
    ctx->scratch_reset();
    const Params p = split_params(c, params);
    const int64_t n = c.num_nodes;
    const int Lg = c.num_gcn_layers, H = c.rnn_hidden;
    const int lstm = c.rnn_kind == REINC_RNN_LSTM;
    const float *nof = nullptr;
    // With loss rows set (a node mini-batch, numbered first) the last GCN layer and the recurrent cell are computed
    // on those rows only (see place_rows).
    const int64_t nt = ctx->top_rows();
    place_rows(ctx, s);
    // the degree scales of a batch of timesteps, next to each other, for a layer that works on its first rows only
    float *q_rows = nullptr;
    if (c.agg_kind != REINC_AGG_SUM) {
        int64_t most = 0;
        for (int l = 1; l <= Lg; ++l)
            if (ctx->rows_of_layer(l) < n && !transform_first(c, l)) most = std::max(most, ctx->rows_of_layer(l));
        if (most > 0) {
            q_rows = static_cast<float *>(ctx->scratch(uint64_t(std::min<int32_t>(L, ctx->max_batch)) * most * 4));
            if (!q_rows) return ctx->fail(REINC_E_NOMEM, "arena exhausted: no room for a batch's degree scales");
        }
    }
    // Layer by layer over batches of timesteps: the dense steps see all timesteps of a batch as one tall matrix
    // (one launch instead of one per timestep), the aggregation of a layer takes the batch's snapshots in one
    // launch; only the layer-1 sums (a chain over snapshots) and the recurrent cell (a chain over time) go
    // timestep by timestep.
    std::vector<const float *> s1(L), q(L), ql(L), Hp(L), Sp(L), Hout(L);
    for (int32_t lo = 0; lo < L; lo += ctx->max_batch) {
        const int32_t hi = std::min(L, lo + ctx->max_batch) - 1;
        for (int32_t i = lo; i <= hi; ++i) {
            REINC_TRY(ensure_layer1(ctx, t0 + i, s));
            s1[i] = ctx->gcache[t0 + i];
            q[i] = ctx->snaps[t0 + i].q;
        }
        for (int l = 1; l <= Lg; ++l) {
            // rows of H^l that anything reads: all of them, or (a node batch) the first nl; the layers below the last
            // keep full-height slices, so with nl < n their timesteps are not adjacent and go one by one
            const int64_t nl = ctx->rows_of_layer(l);
            if (transform_first(c, l)) {
                // Z = H^{l-1} W_l for all timesteps of the batch as one tall matrix (every row of H^{l-1} that exists: the
                // rows are sources), then H^l = ReLU(Q (A + sI) P Z + b_l) straight out of the aggregation kernel
                const int64_t nz = ctx->rows_of_layer(l - 1);
                for (int32_t i = lo; i <= hi; ++i) {
                    Sp[i] = ctx->local[i].H[l - 1];
                    Hout[i] = ctx->local[i].S[l];
                }
                REINC_TRY(for_runs(lo, hi, nz, {Strip{Sp.data(), c.dims[l - 1]}, Strip{Hout.data(), int64_t(s_width_floats(c, l))}},
                                   [&](int i0, int len) {
                                       gemm_rows(ctx, s, (const void *)Sp[i0], 0, nz * len, c.dims[l - 1], c.dims[l], nof, p.W[l], 0,
                                                 c.dims[l], nof, 0, nof, nof, const_cast<float *>(Hout[i0]));
                                       return REINC_OK;
                                   }));
                AggBatch batch;
                batch.count = hi - lo + 1;
                for (int32_t i = lo; i <= hi; ++i) {
                    const Snapshot &sn = ctx->snaps[t0 + i];
                    LocalStep &st = ctx->local[i];
                    AggItem &it = batch.item[i - lo];
                    it = AggItem{sn.row_ptr, sn.col, st.S[l], sn.p, sn.q, nullptr, nullptr, st.H[l], sn.long_rows, sn.n_long_rows};
                    it.bias = p.b[l];
                    it.relu = 1;
                    if (nl < n)
                        it.row_limit = nl;  // rows [0, nl) as they come (the last layer's H has nt rows per timestep)
                    else
                        it.order = sn.row_order;
                }
                aggregate_full_batch(ctx, batch, 0, c.dims[l], c.self_loop, s, nl);
                continue;
            }
            if (l >= 2) {
                AggBatch batch;
                batch.count = hi - lo + 1;
                for (int32_t i = lo; i <= hi; ++i) {
                    const Snapshot &sn = ctx->snaps[t0 + i];
                    LocalStep &st = ctx->local[i];
                    batch.item[i - lo] = AggItem{sn.row_ptr, sn.col, st.H[l - 1], sn.p, nullptr, nullptr, nullptr, st.S[l], sn.long_rows,
                                                 sn.n_long_rows};
                    if (nl < n)
                        batch.item[i - lo].row_limit = nl;  // rows [0, nl) as they come (the last layer's S has nt rows per timestep)
                    else
                        batch.item[i - lo].order = sn.row_order;
                }
                aggregate_full_batch(ctx, batch, 0, c.dims[l - 1], c.self_loop, s, nl);
            }
            for (int32_t i = lo; i <= hi; ++i) {
                Sp[i] = l == 1 ? s1[i] : ctx->local[i].S[l];
                Hout[i] = ctx->local[i].H[l];
                ql[i] = q[i];
            }
            const bool has_q = q[lo] != nullptr;
            if (has_q && nl < n && q_rows) {
                ScaleTable tab{};
                for (int32_t i = lo; i <= hi; ++i) {
                    tab.src[i - lo] = q[i];
                    ql[i] = q_rows + int64_t(i - lo) * nl;
                }
                gather_scales<<<dim3(unsigned((nl + 255) / 256), unsigned(hi - lo + 1)), 256, 0, s>>>(tab, nl, q_rows);
            }
            // (the last layer works on the top rows; with Lg == 1 its input, the cached sums, and the degree scales
            // keep the full height, so a batch's timesteps are not adjacent there and go one by one)
            REINC_TRY(for_runs(lo, hi, nl, {Strip{Sp.data(), c.dims[l - 1]}, Strip{Hout.data(), c.dims[l]},
                                            Strip{has_q ? ql.data() : nullptr, 1}},
                               [&](int i0, int len) {
                                   gemm_rows(ctx, s, (const void *)Sp[i0], 0, nl * len, c.dims[l - 1], c.dims[l], ql[i0], p.W[l], 0,
                                             c.dims[l], p.b[l], 1, nof, nof, const_cast<float *>(Hout[i0]));
                                   return REINC_OK;
                               }));
        }
        for (int32_t i = lo; i <= hi; ++i) {
            LocalStep &st = ctx->local[i];
            const LocalStep *pv = i ? &ctx->local[i - 1] : nullptr;
            const float *hp = pv ? (const float *)pv->h : nof;
            rnn_fused(ctx, s, lstm, (const float *)st.H[Lg], nof, nt, c.dims[Lg], H, hp, hp, pv ? (const float *)pv->c : nof,
                      p.W_i, p.W_h, p.b_i, p.b_h, st.h, st.c, st.saved);
        }
    }
    const LocalStep &last = ctx->local[L - 1];
    if (target) launch_mse(last.h, target, ctx->counted_rows() * H, ctx->loss_partial, loss_out, s);
    if (h_last) REINC_HIP(ctx, hipMemcpyAsync(h_last, last.h, uint64_t(nt) * H * 4, hipMemcpyDeviceToDevice, s));
    REINC_HIP(ctx, hipGetLastError());
    ctx->local_valid = true;
    ctx->local_t0 = t0;
    ctx->local_len = L;
    return REINC_OK;
}

int reinc_backward_window(reinc_ctx *ctx, int32_t t0, int32_t L, const float *params, const float *target, float *grads,
                          void *stream)
{
    if (!ctx) return REINC_E_ARG;
    REINC_TRY(check_window(ctx, t0, L));
    if (!params || !target || !grads) return ctx->fail(REINC_E_ARG, "null params, target or grads");
    if (!ctx->local_valid || ctx->local_kind != 0 || ctx->local_t0 != t0 || ctx->local_len != L)
        return ctx->fail(REINC_E_STATE, "backward needs the forward pass of the same window [%d, %d) first", t0, t0 + L);
    const reinc_config &c = ctx->cfg;
    hipStream_t s = as_stream(stream);
    REINC_HIP(ctx, hipSetDevice(c.device));
    const Params p = split_params(c, params);
    Params gp = split_params(c, grads);
    const int64_t n = c.num_nodes;
    const int64_t nt = ctx->top_rows();  // rows of the last GCN layer and of the recurrent cell (see place_rows)
    if (ctx->local_top != nt) return ctx->fail(REINC_E_STATE, "the loss rows changed since the forward pass of this window");
    for (int l = 1; l <= c.num_gcn_layers; ++l)
        if (ctx->local_rows[l] != ctx->rows_of_layer(l))
            return ctx->fail(REINC_E_STATE, "the rows of layer %d changed since the forward pass of this window", l);
    const int Lg = c.num_gcn_layers, H = c.rnn_hidden;
    const int lstm = c.rnn_kind == REINC_RNN_LSTM;
    const int KH = (lstm ? 4 : 3) * H;
    int maxd = H;
    for (int l = 0; l <= Lg; ++l) maxd = std::max(maxd, c.dims[l]);

    // Scratch.  The recurrent chain runs timestep by timestep; everything else of the backward pass is done for a
    // batch of B timesteps at a time (tall matrices, one aggregation launch per layer), which needs the gate and
    // layer gradients of B timesteps at once.  B is the largest depth (at most the window, at most kMaxAggBatch)
    // whose buffers fit the free part of the arena.
    ctx->scratch_reset();
    auto f32 = [&](uint64_t count) { return static_cast<float *>(ctx->scratch(count * 4)); };
    float *dh = f32(uint64_t(n) * H), *dh2 = f32(uint64_t(n) * H);
    float *dc = lstm ? f32(uint64_t(n) * H) : nullptr, *dc2 = lstm ? f32(uint64_t(n) * H) : nullptr;
    bool ok = dh && dh2 && (!lstm || (dc && dc2));
    const uint64_t free_bytes = ok ? ctx->top - ctx->bottom : 0;
    auto batch_bytes = [&](int B) {
        const uint64_t rows = uint64_t(B) * uint64_t(n);
        uint64_t b = align256(rows * KH * 4) * (lstm ? 1 : 2) + 3 * align256(rows * maxd * 4);
        b += align256(reduce_partial_bytes(int64_t(rows), c.dims[Lg], KH)) + align256(reduce_partial_bytes(int64_t(rows), H, KH));
        for (int l = 1; l <= Lg; ++l) b += align256(reduce_partial_bytes(int64_t(rows), c.dims[l - 1], c.dims[l]));
        return b + align256(column_sums_bytes(maxd));
    };
    int B = std::min<int>(L, ctx->max_batch);
    while (B > 1 && batch_bytes(B) > free_bytes) --B;
    if (!ok || batch_bytes(B) > free_bytes) {
        ctx->scratch_reset();
        return ctx->fail(REINC_E_NOMEM, "arena exhausted: no room for the backward scratch buffers");
    }
    const int64_t rowsB = int64_t(B) * n;
    const int64_t rowsT = int64_t(B) * nt;  // rows of a batch of timesteps in the top quantities
    float *dgi = f32(uint64_t(rowsB) * KH);
    float *dgh = lstm ? dgi : f32(uint64_t(rowsB) * KH);
    float *dz = f32(uint64_t(rowsB) * maxd), *dz2 = f32(uint64_t(rowsB) * maxd), *dagg = f32(uint64_t(rowsB) * maxd);
    // one set of partial slabs per weight matrix: they collect all batches and are reduced once at the end
    float *part_wi = static_cast<float *>(ctx->scratch(reduce_partial_bytes(rowsT, c.dims[Lg], KH)));
    float *part_wh = static_cast<float *>(ctx->scratch(reduce_partial_bytes(rowsT, H, KH)));
    float *part_w[REINC_MAX_GCN_LAYERS + 1] = {};
    bool part_ok = part_wi && part_wh;
    auto layer_rows = [&](int l) { return l == Lg && !transform_first(c, l) ? rowsT : rowsB; };  // rows its weight gradient sums over
    for (int l = 1; l <= Lg; ++l) {
        part_w[l] = static_cast<float *>(ctx->scratch(reduce_partial_bytes(layer_rows(l), c.dims[l - 1], c.dims[l])));
        part_ok = part_ok && part_w[l];
    }
    float *colsum = static_cast<float *>(ctx->scratch(column_sums_bytes(maxd)));
    part_ok = part_ok && colsum;
    // the degree scales of a batch of timesteps, next to each other, for a layer that works on its first rows only
    float *q_rows = nullptr;
    if (c.agg_kind != REINC_AGG_SUM) {
        int64_t most = 0;
        for (int l = 1; l <= Lg; ++l)
            if (ctx->rows_of_layer(l) < n && !transform_first(c, l)) most = std::max(most, ctx->rows_of_layer(l));
        if (most > 0) {
            q_rows = static_cast<float *>(ctx->scratch(uint64_t(B) * most * 4));
            part_ok = part_ok && q_rows;
        }
    }
    if (!dgi || !dgh || !dz || !dz2 || !dagg || !part_ok) {
        ctx->scratch_reset();
        return ctx->fail(REINC_E_NOMEM, "arena exhausted: no room for the backward scratch buffers");
    }
    launch_fill_f32(grads, p.count, 0.0f, s);
    launch_mse_grad(ctx->local[L - 1].h, target, ctx->counted_rows() * H, nt * H, dh, s);
    const float *dc_in = nullptr;  // zero at the last step
    const float *nof = nullptr;
    std::vector<const float *> s1(L), q(L), ql(L), Ap(L), Mp(L);
    // The partial slabs of a weight always belong to the same number of rows (B timesteps): a shorter last batch
    // uses the chunk geometry of a full one, so that every batch adds into the same slabs.
    auto reduce = [&](const float *A, int lda, const float *rs, const float *G, int ldg, int64_t rows, int64_t rows_geom, int K, int M,
                      float *part, int accumulate) { gemm_reduce(ctx, s, A, lda, rs, G, ldg, rows, rows_geom, K, M, part, accumulate); };
    bool first_batch = true;
    for (int32_t hi = L - 1; hi >= 0;) {
        const int32_t lo = std::max(0, hi - B + 1);
        const int nb = hi - lo + 1;
        // the recurrent chain of the batch, last timestep first
        for (int32_t i = hi; i >= lo; --i) {
            const LocalStep &st = ctx->local[i];
            const LocalStep *pv = i ? &ctx->local[i - 1] : nullptr;
            float *dgi_i = dgi + int64_t(i - lo) * nt * KH, *dgh_i = dgh + int64_t(i - lo) * nt * KH;
            rnn_backward_elem(ctx, s, lstm, nt, H, (const float *)dh, dc_in, (const float *)st.saved,
                              pv ? (const float *)pv->h : nof, pv ? (const float *)pv->c : nof, (const float *)st.c, dgi_i, dgh_i,
                              dh2, dc2);
            if (i > 0) {  // gradient w.r.t. h_{t-1}
                gemm_rows(ctx, s, (const void *)dgh_i, 0, nt, KH, H, nof, p.W_h, 1, KH, nof, 0, lstm ? nof : (const float *)dh2,
                          nof, dh);
                if (lstm) {
                    std::swap(dc, dc2);  // dc now holds the gradient w.r.t. c_{t-1}; dc2 is free for the next step
                    dc_in = dc;
                }
            }
        }
        for (int32_t i = lo; i <= hi; ++i) {
            s1[i] = ctx->gcache[t0 + i];
            q[i] = ctx->snaps[t0 + i].q;
        }
        const bool has_q = q[lo] != nullptr;
        const int acc0 = first_batch ? 0 : 1;
        const int dl = c.dims[Lg];
        // recurrent weights: x_t = H^{Lg}_t against the x-side gate gradients, h_{t-1} against the h-side ones
        for (int32_t i = lo; i <= hi; ++i) {
            Ap[i] = ctx->local[i].H[Lg];
            Mp[i] = i ? ctx->local[i - 1].h : ctx->zero_state;
        }
        int calls = 0;
        REINC_TRY(for_runs(lo, hi, nt, {Strip{Ap.data(), dl}}, [&](int i0, int len) {
            reduce(Ap[i0], dl, nof, dgi + int64_t(i0 - lo) * nt * KH, KH, nt * len, rowsT, dl, KH, part_wi, acc0 | (calls++ > 0));
            return REINC_OK;
        }));
        calls = 0;
        REINC_TRY(for_runs(lo, hi, nt, {Strip{Mp.data(), H}}, [&](int i0, int len) {
            reduce(Mp[i0], H, nof, dgh + int64_t(i0 - lo) * nt * KH, KH, nt * len, rowsT, H, KH, part_wh, acc0 | (calls++ > 0));
            return REINC_OK;
        }));
        // gradient w.r.t. the last GCN layer's pre-activation, all timesteps of the batch
        REINC_TRY(for_runs(lo, hi, nt, {Strip{Ap.data(), dl}}, [&](int i0, int len) {
            gemm_rows(ctx, s, (const void *)(dgi + int64_t(i0 - lo) * nt * KH), 0, nt * len, KH, dl, nof, p.W_i, 1, KH, nof, 0, nof,
                      Ap[i0], dz + int64_t(i0 - lo) * nt * dl);
            return REINC_OK;
        }));
        for (int l = Lg; l >= 1; --l) {
            const int din = c.dims[l - 1], dout = c.dims[l];
            calls = 0;
            // dz holds the gradients of layer l's pre-activations: nl rows per timestep, the timesteps next to each other.
            // np: the rows of layer l - 1 that anything reads (the sources of the rows of layer l lie among them).
            const int64_t nl = ctx->rows_of_layer(l);
            const int64_t np = l > 1 ? ctx->rows_of_layer(l - 1) : n;
            const bool part_l = nl < n;  // only some rows exist: what reads every row is given zeros for the others
            auto adjoint_item = [&](AggItem &it, const Snapshot &sn) {  // its output rows are the sources
                if (np < n)
                    it.row_limit = np;
                else
                    it.order = sn.col_order;
            };
            if (transform_first(c, l)) {
                // H^l = ReLU(Q (A + sI) P Z + b_l), Z = H^{l-1} W_l:  db_l = column sums of dz;  dZ = P (A + sI)^T Q dz (the
                // adjoint gather, dout wide);  dW_l = H^{l-1}^T dZ;  dz of layer l-1 = (dZ W_l^T) masked by H^{l-1} > 0
                launch_column_sums(dz, nl * nb, dout, colsum, const_cast<float *>(gp.b[l]), 1, s);
                const float *dz_full = dz;
                if (part_l) {  // the adjoint reads every row: the rows that are not computed are zero
                    launch_fill_f32(dagg, int64_t(nb) * n * dout, 0.0f, s);
                    for (int32_t i = lo; i <= hi; ++i)
                        REINC_HIP(ctx, hipMemcpyAsync(dagg + int64_t(i - lo) * n * dout, dz + int64_t(i - lo) * nl * dout,
                                                      uint64_t(nl) * dout * 4, hipMemcpyDeviceToDevice, s));
                    dz_full = dagg;
                }
                AggBatch batch;
                batch.count = nb;
                for (int32_t i = lo; i <= hi; ++i) {
                    const Snapshot &sn = ctx->snaps[t0 + i];
                    batch.item[i - lo] = AggItem{sn.col_ptr, sn.row, dz_full + int64_t(i - lo) * n * dout, sn.q, sn.p, nullptr, nullptr,
                                                 dz2 + int64_t(i - lo) * np * dout, sn.long_cols, sn.n_long_cols};
                    adjoint_item(batch.item[i - lo], sn);
                }
                aggregate_full_batch(ctx, batch, 0, dout, c.self_loop, s, np);
                for (int32_t i = lo; i <= hi; ++i) Ap[i] = ctx->local[i].H[l - 1];
                REINC_TRY(for_runs(lo, hi, np, {Strip{Ap.data(), din}}, [&](int i0, int len) {
                    reduce(Ap[i0], din, nof, dz2 + int64_t(i0 - lo) * np * dout, dout, np * len, rowsB, din, dout, part_w[l],
                           acc0 | (calls++ > 0));
                    gemm_rows(ctx, s, (const void *)(dz2 + int64_t(i0 - lo) * np * dout), 0, np * len, dout, din, nof, p.W[l], 1, dout, nof,
                              0, nof, Ap[i0], (part_l ? dz : dagg) + int64_t(i0 - lo) * np * din);
                    return REINC_OK;
                }));
                if (!part_l) std::swap(dz, dagg);  // (else dz itself received the result: dagg held its zero-padded copy)
                continue;
            }
            for (int32_t i = lo; i <= hi; ++i) {
                Ap[i] = l == 1 ? s1[i] : ctx->local[i].S[l];
                ql[i] = q[i];
            }
            if (has_q && part_l && q_rows) {
                ScaleTable tab{};
                for (int32_t i = lo; i <= hi; ++i) {
                    tab.src[i - lo] = q[i];
                    ql[i] = q_rows + int64_t(i - lo) * nl;
                }
                gather_scales<<<dim3(unsigned((nl + 255) / 256), unsigned(nb)), 256, 0, s>>>(tab, nl, q_rows);
            }
            REINC_TRY(for_runs(lo, hi, nl, {Strip{Ap.data(), din}, Strip{has_q ? ql.data() : nullptr, 1}},
                               [&](int i0, int len) {
                                   reduce(Ap[i0], din, ql[i0], dz + int64_t(i0 - lo) * nl * dout, dout, nl * len, l == Lg ? rowsT : rowsB,
                                          din, dout, part_w[l], acc0 | (calls++ > 0));
                                   return REINC_OK;
                               }));
            if (l > 1) {
                if (part_l) {
                    // the adjoint aggregation below reads every row of dagg (full height): the rows that are not computed
                    // are zero
                    launch_fill_f32(dagg, int64_t(nb) * n * din, 0.0f, s);
                    for (int32_t i = lo; i <= hi; ++i)
                        gemm_rows(ctx, s, (const void *)(dz + int64_t(i - lo) * nl * dout), 0, nl, dout, din, nof, p.W[l], 1, dout, nof, 0,
                                  nof, nof, dagg + int64_t(i - lo) * n * din);
                } else
                    gemm_rows(ctx, s, (const void *)dz, 0, n * nb, dout, din, nof, p.W[l], 1, dout, nof, 0, nof, nof, dagg);
                AggBatch batch;
                batch.count = nb;
                for (int32_t i = lo; i <= hi; ++i) {
                    const Snapshot &sn = ctx->snaps[t0 + i];
                    batch.item[i - lo] = AggItem{sn.col_ptr, sn.row, dagg + int64_t(i - lo) * n * din, sn.q, sn.p,
                                                 ctx->local[i].H[l - 1], nullptr, dz2 + int64_t(i - lo) * np * din, sn.long_cols,
                                                 sn.n_long_cols};
                    adjoint_item(batch.item[i - lo], sn);
                }
                aggregate_full_batch(ctx, batch, 0, din, c.self_loop, s, np);
                std::swap(dz, dz2);
            }
        }
        first_batch = false;
        hi = lo - 1;
    }
    launch_reduce_partials(part_wi, rowsT, c.dims[Lg], KH, const_cast<float *>(gp.W_i), const_cast<float *>(gp.b_i), s);
    launch_reduce_partials(part_wh, rowsT, H, KH, const_cast<float *>(gp.W_h), const_cast<float *>(gp.b_h), s);
    for (int l = 1; l <= Lg; ++l)  // (the bias gradient of a transform-first layer is not the slabs' column sum: see above)
        launch_reduce_partials(part_w[l], layer_rows(l), c.dims[l - 1], c.dims[l], const_cast<float *>(gp.W[l]),
                               transform_first(c, l) ? nullptr : const_cast<float *>(gp.b[l]), s);
    REINC_HIP(ctx, hipGetLastError());
    return REINC_OK;
}

// ---- the integrated model (Section 2.1: graph operations on x_t and h_{t-1} inside the recurrent gates; Section 3.1:
// both are aggregated once per timestep and shared by all gates).  params: W_i [dims[0], K*H], W_h [H, K*H], b_i, b_h.
int reinc_forward_window_integrated(reinc_ctx *ctx, int32_t t0, int32_t L, const float *params, const float *target,
                                    float *loss_out, float *h_last, void *stream)
{
    if (!ctx) return REINC_E_ARG;
    REINC_TRY(check_window(ctx, t0, L));
    // A batch context computes timestep i on the nodes within L - 1 - i hops of the batch (nothing else reaches the
    // batch rows by the window's end); its cached input sums must hold the rows of the first timestep.  Sums cached with
    // fewer rows (by the stacked model, or by a shorter window) are dropped.
    const int64_t need_rows = ctx->integrated_rows(L, 0);
    if (ctx->cache_rows > 0 && ctx->cache_rows < need_rows) {
        REINC_TRY(reinc_cache_clear(ctx));
        ctx->cache_rows = need_rows < ctx->cfg.num_nodes ? need_rows : 0;
    }
    if (!params) return ctx->fail(REINC_E_ARG, "null parameter vector");
    if (target && !loss_out) return ctx->fail(REINC_E_ARG, "a target needs loss_out");
    const reinc_config &c = ctx->cfg;
    const int H = c.rnn_hidden;
    if (!agg_width_supported(H, 0))
        return ctx->fail(REINC_E_UNSUPPORTED, "hidden width %d: row bytes must be a power of two in [16, 1024]", H);
    hipStream_t s = as_stream(stream);
    REINC_HIP(ctx, hipSetDevice(c.device));
    ctx->local_valid = false;
    REINC_TRY(begin_budgeted_window(ctx, t0, L));
    REINC_TRY(ensure_local_integrated(ctx, L, s));
    ctx->scratch_reset();
    const int64_t n = c.num_nodes;
    const int lstm = c.rnn_kind == REINC_RNN_LSTM;
    const int64_t KH = int64_t(lstm ? 4 : 3) * H;
    const float *W_i = params, *W_h = W_i + int64_t(c.dims[0]) * KH, *b_i = W_h + int64_t(H) * KH, *b_h = b_i + KH;
    const float *nof = nullptr;
    ctx->step_rows.assign(size_t(L), n);
    for (int32_t i = 0; i < L; ++i) {
        const int32_t t = t0 + i;
        REINC_TRY(ensure_layer1(ctx, t, s));  // Agg(X_t): from the global cache, by Eq. 2, or from scratch
        const Snapshot &sn = ctx->snaps[t];
        LocalStep &st = ctx->local[i];
        const LocalStep *pv = i ? &ctx->local[i - 1] : nullptr;
        const int64_t ni = ctx->integrated_rows(L, i);  // (the sources of these rows lie among the rows of timestep i - 1)
        ctx->step_rows[size_t(i)] = ni;
        if (pv) {  // Agg(h_{t-1}) over snapshot t; at the first timestep the state, and with it the aggregate, is zero
            AggBatch batch;
            batch.count = 1;
            batch.item[0] = AggItem{sn.row_ptr, sn.col, pv->h, sn.p, sn.q, nullptr, nullptr, st.S[1], sn.long_rows, sn.n_long_rows};
            if (ni < n)
                batch.item[0].row_limit = ni;
            else
                batch.item[0].order = sn.row_order;
            aggregate_full_batch(ctx, batch, 0, H, c.self_loop, s, ni);
        }
        rnn_fused(ctx, s, lstm, (const float *)ctx->gcache[t], (const float *)sn.q, ni, c.dims[0], H,
                  pv ? (const float *)st.S[1] : nof, pv ? (const float *)pv->h : nof, pv ? (const float *)pv->c : nof, W_i, W_h,
                  b_i, b_h, st.h, st.c, st.saved);
    }
    const LocalStep &last = ctx->local[L - 1];
    const int64_t n_last = ctx->step_rows[size_t(L - 1)];  // (a batch context: the loss rows)
    if (target) launch_mse(last.h, target, ctx->counted_rows() * H, ctx->loss_partial, loss_out, s);
    if (h_last) REINC_HIP(ctx, hipMemcpyAsync(h_last, last.h, uint64_t(n_last) * H * 4, hipMemcpyDeviceToDevice, s));
    REINC_HIP(ctx, hipGetLastError());
    ctx->local_valid = true;
    ctx->local_t0 = t0;
    ctx->local_len = L;
    return REINC_OK;
}

int reinc_backward_window_integrated(reinc_ctx *ctx, int32_t t0, int32_t L, const float *params, const float *target,
                                     float *grads, void *stream)
{
    if (!ctx) return REINC_E_ARG;
    REINC_TRY(check_window(ctx, t0, L));
    if (!params || !target || !grads) return ctx->fail(REINC_E_ARG, "null params, target or grads");
    if (!ctx->local_valid || ctx->local_kind != 1 || ctx->local_t0 != t0 || ctx->local_len != L)
        return ctx->fail(REINC_E_STATE, "backward needs the integrated forward pass of the same window [%d, %d) first", t0, t0 + L);
    const reinc_config &c = ctx->cfg;
    hipStream_t s = as_stream(stream);
    REINC_HIP(ctx, hipSetDevice(c.device));
    const int64_t n = c.num_nodes;
    const int H = c.rnn_hidden, d0 = c.dims[0];
    const int lstm = c.rnn_kind == REINC_RNN_LSTM;
    const int KH = (lstm ? 4 : 3) * H;
    const float *W_h = params + int64_t(d0) * KH;
    float *gW_i = grads, *gW_h = gW_i + int64_t(d0) * KH, *gb_i = gW_h + int64_t(H) * KH, *gb_h = gb_i + KH;
    const int64_t count = int64_t(d0 + H + 2) * KH;

    ctx->scratch_reset();
    auto f32 = [&](uint64_t cnt) { return static_cast<float *>(ctx->scratch(cnt * 4)); };
    float *dh = f32(uint64_t(n) * H), *dh2 = f32(uint64_t(n) * H), *dah = f32(uint64_t(n) * H);
    float *dc = lstm ? f32(uint64_t(n) * H) : nullptr, *dc2 = lstm ? f32(uint64_t(n) * H) : nullptr;
    bool ok = dh && dh2 && dah && (!lstm || (dc && dc2));
    const uint64_t free_bytes = ok ? ctx->top - ctx->bottom : 0;
    auto batch_bytes = [&](int B) {
        const uint64_t rows = uint64_t(B) * uint64_t(n);
        return align256(rows * KH * 4) * (lstm ? 1 : 2) + align256(reduce_partial_bytes(int64_t(rows), d0, KH)) +
               align256(reduce_partial_bytes(int64_t(rows), H, KH));
    };
    int B = std::min<int>(L, ctx->max_batch);
    while (B > 1 && batch_bytes(B) > free_bytes) --B;
    if (!ok || batch_bytes(B) > free_bytes) {
        ctx->scratch_reset();
        return ctx->fail(REINC_E_NOMEM, "arena exhausted: no room for the backward scratch buffers");
    }
    const int64_t rowsB = int64_t(B) * n;
    float *dgi = f32(uint64_t(rowsB) * KH);
    float *dgh = lstm ? dgi : f32(uint64_t(rowsB) * KH);
    float *part_wi = static_cast<float *>(ctx->scratch(reduce_partial_bytes(rowsB, d0, KH)));
    float *part_wh = static_cast<float *>(ctx->scratch(reduce_partial_bytes(rowsB, H, KH)));
    if (!dgi || !dgh || !part_wi || !part_wh) {
        ctx->scratch_reset();
        return ctx->fail(REINC_E_NOMEM, "arena exhausted: no room for the backward scratch buffers");
    }
    launch_fill_f32(grads, count, 0.0f, s);
    launch_mse_grad(ctx->local[L - 1].h, target, ctx->counted_rows() * H, n * H, dh, s);
    // A batch context computed timestep i on its first step_rows[i] rows (non-increasing in i).  Going back in time the
    // row count only grows, so whatever a step leaves beyond its rows -- the gradient w.r.t. the aggregated state, the
    // carried state gradients -- is still the zero it starts as: what reads every row finds zeros there.
    const std::vector<int64_t> &rows_of = ctx->step_rows;
    if (int32_t(rows_of.size()) != L) return ctx->fail(REINC_E_STATE, "the forward pass left no row counts for this window");
    const bool part = rows_of[size_t(L - 1)] < n;
    if (part) {
        launch_fill_f32(dah, n * H, 0.0f, s);
        launch_fill_f32(dh2, n * H, 0.0f, s);
        if (lstm) {
            launch_fill_f32(dc, n * H, 0.0f, s);
            launch_fill_f32(dc2, n * H, 0.0f, s);
        }
    }
    const float *dc_in = nullptr;
    const float *nof = nullptr;
    std::vector<const float *> s1(L), q(L), ah(L);
    bool first_batch = true;
    for (int32_t hi = L - 1; hi >= 0;) {
        const int32_t lo = std::max(0, hi - B + 1);
        for (int32_t i = hi; i >= lo; --i) {
            const Snapshot &sn = ctx->snaps[t0 + i];
            const LocalStep &st = ctx->local[i];
            const LocalStep *pv = i ? &ctx->local[i - 1] : nullptr;
            const int64_t ni = rows_of[size_t(i)];
            float *dgi_i = dgi + int64_t(i - lo) * n * KH, *dgh_i = dgh + int64_t(i - lo) * n * KH;
            rnn_backward_elem(ctx, s, lstm, ni, H, (const float *)dh, dc_in, (const float *)st.saved,
                              pv ? (const float *)pv->h : nof, pv ? (const float *)pv->c : nof, (const float *)st.c, dgi_i, dgh_i,
                              dh2, dc2);
            if (i > 0) {
                // gradient w.r.t. Agg(h_{t-1}), then through the adjoint of the aggregation, plus the carry path
                const int64_t np = rows_of[size_t(i - 1)];  // rows of h_{t-1} that exist: the output rows of the adjoint
                gemm_rows(ctx, s, (const void *)dgh_i, 0, ni, KH, H, nof, W_h, 1, KH, nof, 0, nof, nof, dah);
                AggBatch batch;
                batch.count = 1;
                batch.item[0] = AggItem{sn.col_ptr, sn.row, dah, sn.q, sn.p, nullptr, lstm ? nof : (const float *)dh2, dh,
                                        sn.long_cols, sn.n_long_cols};
                if (np < n)
                    batch.item[0].row_limit = np;
                else
                    batch.item[0].order = sn.col_order;
                aggregate_full_batch(ctx, batch, 0, H, c.self_loop, s, np);
                if (lstm) {
                    std::swap(dc, dc2);
                    dc_in = dc;
                }
            }
        }
        for (int32_t i = lo; i <= hi; ++i) {
            s1[i] = ctx->gcache[t0 + i];
            q[i] = ctx->snaps[t0 + i].q;
            ah[i] = ctx->local[i].S[1];
        }
        const bool has_q = q[lo] != nullptr;
        const int acc0 = first_batch ? 0 : 1;
        int calls = 0;
        if (part) {
            // every timestep has its own row count: one reduction each, over the rows that exist
            for (int32_t i = lo; i <= hi; ++i, ++calls) {
                const int64_t ni = rows_of[size_t(i)];
                gemm_reduce(ctx, s, s1[i], d0, q[i], (const float *)(dgi + int64_t(i - lo) * n * KH), KH, ni, rowsB, d0, KH, part_wi,
                            acc0 | (calls > 0));
                gemm_reduce(ctx, s, ah[i], H, nof, (const float *)(dgh + int64_t(i - lo) * n * KH), KH, ni, rowsB, H, KH, part_wh,
                            acc0 | (calls > 0));
            }
            first_batch = false;
            hi = lo - 1;
            continue;
        }
        REINC_TRY(for_runs(lo, hi, n, {Strip{s1.data(), d0}, Strip{has_q ? q.data() : nullptr, 1}}, [&](int i0, int len) {
            gemm_reduce(ctx, s, s1[i0], d0, q[i0], (const float *)(dgi + int64_t(i0 - lo) * n * KH), KH, n * len, rowsB, d0, KH,
                        part_wi, acc0 | (calls++ > 0));
            return REINC_OK;
        }));
        calls = 0;
        REINC_TRY(for_runs(lo, hi, n, {Strip{ah.data(), H}}, [&](int i0, int len) {
            gemm_reduce(ctx, s, ah[i0], H, nof, (const float *)(dgh + int64_t(i0 - lo) * n * KH), KH, n * len, rowsB, H, KH, part_wh,
                        acc0 | (calls++ > 0));
            return REINC_OK;
        }));
        first_batch = false;
        hi = lo - 1;
    }
    launch_reduce_partials(part_wi, rowsB, d0, KH, gW_i, gb_i, s);
    launch_reduce_partials(part_wh, rowsB, H, KH, gW_h, gb_h, s);
    REINC_HIP(ctx, hipGetLastError());
    return REINC_OK;
}

int reinc_cache_clear(reinc_ctx *ctx)
{
    if (!ctx) return REINC_E_ARG;
    if (ctx->gpolicy) {
        // every buffer returns to the pool; the pool itself stays
        ctx->gpolicy->clear();
        ctx->pool_free = ctx->pool;
        ctx->pending.clear();
        ctx->expired_pending.clear();
        std::fill(ctx->gcache.begin(), ctx->gcache.end(), nullptr);
        ctx->local_valid = false;
        ctx->sync_policy_stats();
        return REINC_OK;
    }
    // cached sums live in the persistent region and cannot be returned piecemeal: forget them and let the
    // next windows recompute into fresh slots only if every slot sits at the end of the region
    uint64_t lowest = ctx->bottom;
    bool any = false;
    for (float *p : ctx->gcache)
        if (p) {
            any = true;
            lowest = std::min<uint64_t>(lowest, uint64_t(reinterpret_cast<char *>(p) - ctx->base));
        }
    if (any) {
        // release the tail of the persistent region when nothing else was allocated after the first slot
        const uint64_t slot = (uint64_t(ctx->cached_rows()) * ctx->cfg.dims[0] * 4 + 255) & ~uint64_t(255);
        uint64_t count = 0;
        for (float *p : ctx->gcache) count += p != nullptr;
        if (lowest + count * slot == ctx->bottom) ctx->bottom = lowest;
    }
    std::fill(ctx->gcache.begin(), ctx->gcache.end(), nullptr);
    ctx->local_valid = false;
    return REINC_OK;
}

int reinc_cache_configure(reinc_ctx *ctx, int32_t policy, int64_t budget_bytes, int32_t window, int32_t stride)
{
    if (!ctx) return REINC_E_ARG;
    if (policy < REINC_POLICY_KEEP_ALL || policy > REINC_POLICY_LFU) return ctx->fail(REINC_E_ARG, "unknown cache policy %d", policy);
    REINC_TRY(reinc_cache_clear(ctx));
    if (policy == REINC_POLICY_KEEP_ALL) {
        // buffers taken for an earlier budget stay in the arena until reinc_reset_derived
        ctx->gpolicy.reset();
        ctx->budget_slots = 0;
        ctx->plan_window = 0;
        ctx->plan_stride = 1;
        return REINC_OK;
    }
    if (budget_bytes < 0 || window < 1 || window > ctx->cfg.num_snapshots || stride < 1)
        return ctx->fail(REINC_E_ARG, "cache budget: need budget_bytes >= 0, 1 <= window <= %d snapshots, stride >= 1",
                         ctx->cfg.num_snapshots);
    const int64_t size = int64_t(aggregate_bytes(ctx->cfg));
    ctx->budget_slots = std::min<int64_t>(budget_bytes / size, ctx->cfg.num_snapshots);  // more can never be held
    ctx->plan_window = window;
    ctx->plan_stride = stride;
    CachePolicy *store = new (std::nothrow) CachePolicy(policy, ctx->budget_slots * size);
    if (!store) return ctx->fail(REINC_E_NOMEM, "out of host memory");
    ctx->gpolicy.reset(store);
    ctx->pool_free = ctx->pool;  // buffers of an earlier budget are reused; more are taken at the next window if needed
    ctx->sync_policy_stats();
    return REINC_OK;
}

int reinc_cache_peek(reinc_ctx *ctx, int32_t t, const float **S_out)
{
    if (!ctx || !S_out) return REINC_E_ARG;
    if (t < 0 || t >= ctx->cfg.num_snapshots) return ctx->fail(REINC_E_ARG, "snapshot index %d out of range", t);
    *S_out = ctx->gcache[t];
    return REINC_OK;
}

}  // extern "C"
