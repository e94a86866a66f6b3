// Dense-step entry points and the window driver with its two caches (paper Section 2.2: a window of L
// consecutive snapshots is one training sample with back-propagation through time; Section 3.3: a global
// cache for the aggregates of the input features, a local cache for per-layer intermediates).
#include <algorithm>

#include "ctx.h"

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

// The window driver spreads independent kernels over up to three side streams (all at the default priority)
// and orders them with events: `to` waits for everything enqueued on `from` so far.
int ensure_side_streams(reinc_ctx *ctx)
{
    for (hipStream_t &st : ctx->side)
        if (!st) REINC_HIP(ctx, hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
    if (ctx->order_events.empty()) {
        ctx->order_events.resize(512);
        for (hipEvent_t &e : ctx->order_events) REINC_HIP(ctx, hipEventCreateWithFlags(&e, hipEventDisableTiming));
    }
    return REINC_OK;
}

int order_after(reinc_ctx *ctx, hipStream_t from, hipStream_t to)
{
    if (from == to) return REINC_OK;
    hipEvent_t e = ctx->order_events[ctx->order_next++ % ctx->order_events.size()];
    REINC_HIP(ctx, hipEventRecord(e, from));
    REINC_HIP(ctx, hipStreamWaitEvent(to, e, 0));
    return REINC_OK;
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

uint64_t local_step_bytes(const reinc_config &c)
{
    const uint64_t n = uint64_t(c.num_nodes);
    uint64_t b = 0;
    for (int l = 1; l <= c.num_gcn_layers; ++l) {
        b += align256(n * c.dims[l] * 4);
        if (l >= 2) b += align256(n * c.dims[l - 1] * 4);
    }
    b += align256(n * c.rnn_hidden * 4);                                     // h
    if (c.rnn_kind == REINC_RNN_LSTM) b += align256(n * c.rnn_hidden * 4);   // c
    b += align256(n * 4 * c.rnn_hidden * 4);                                 // gate values
    return b;
}

// The local cache holds the last `local_reserved` bytes of the arena; it is re-carved when a longer window arrives.
int ensure_local(reinc_ctx *ctx, int32_t L, hipStream_t s)
{
    const reinc_config &c = ctx->cfg;
    if (ctx->local_L >= L && !ctx->local.empty()) return REINC_OK;
    const uint64_t n = uint64_t(c.num_nodes);
    const uint64_t fixed = align256(n * c.rnn_hidden * 4) + align256(loss_partial_bytes());
    const uint64_t need = fixed + uint64_t(L) * local_step_bytes(c);
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
    ctx->zero_state = take(n * c.rnn_hidden * 4);
    ctx->loss_partial = take(loss_partial_bytes());
    ctx->local.assign(L, LocalStep());
    for (int32_t i = 0; i < L; ++i) {
        LocalStep &st = ctx->local[i];
        for (int l = 1; l <= c.num_gcn_layers; ++l) {
            st.H[l] = take(n * c.dims[l] * 4);
            if (l >= 2) st.S[l] = take(n * c.dims[l - 1] * 4);
        }
        st.h = take(n * c.rnn_hidden * 4);
        if (c.rnn_kind == REINC_RNN_LSTM) st.c = take(n * c.rnn_hidden * 4);
        st.saved = take(n * 4 * c.rnn_hidden * 4);
    }
    ctx->local_L = L;
    ctx->local_valid = false;
    ctx->stats.local_bytes = int64_t(need);
    launch_fill_f32(ctx->zero_state, int64_t(n) * c.rnn_hidden, 0.0f, s);
    return REINC_OK;
}

// Makes sure the layer-1 sums of snapshot t are in the global cache.
int ensure_layer1(reinc_ctx *ctx, int32_t t, hipStream_t s)
{
    const reinc_config &c = ctx->cfg;
    if (ctx->gcache[t]) {
        ++ctx->stats.global_hits;
        return REINC_OK;
    }
    const Snapshot &sn = ctx->snaps[t];
    if (!sn.edges_loaded || !sn.feats_loaded)
        return ctx->fail(REINC_E_STATE, "snapshot %d needs its edges and features loaded", t);
    const int32_t d = c.dims[0];
    const int bf16 = c.feat_dtype == REINC_BF16;
    const uint64_t bytes = uint64_t(c.num_nodes) * d * 4;
    ctx->note_derived();
    float *slot = static_cast<float *>(ctx->alloc(bytes));
    if (!slot) return ctx->fail(REINC_E_NOMEM, "arena exhausted: no room for the cached aggregate of snapshot %d", t);
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
            ProfScope prof(ctx, REINC_K_AGG_INC, s);
            launch_incremental(nullptr, c.num_nodes, dl.long_rows, dl.n_long_rows, dl.ent_ptr, dl.ent, pv.x, bf16, pv.p, dl.dY,
                               d, ctx->gcache[t - 1], slot, nullptr, nullptr, s);
        }
        ++ctx->stats.steps_incremental;
        ctx->stats.delta_entries_processed += dl.info.n_entries;
    } else {
        aggregate_full(ctx, sn.row_ptr, sn.col, sn.long_rows, sn.n_long_rows, sn.x, bf16, d, c.self_loop, sn.p, nullptr,
                       nullptr, slot, s);
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
    rnn_fused(ctx, as_stream(stream), int(rnn_kind == REINC_RNN_LSTM), x, n, d_in, H, h_prev, c_prev, W_i, W_h, b_i, b_h,
              h_out, c_out, saved);
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
    for (int l = 1; l < c.num_gcn_layers; ++l)
        if (!agg_width_supported(c.dims[l], 0))
            return ctx->fail(REINC_E_UNSUPPORTED, "layer width %d: row bytes must be a power of two in [16, 1024]", c.dims[l]);
    hipStream_t s = as_stream(stream);
    REINC_HIP(ctx, hipSetDevice(c.device));
    ctx->local_valid = false;
    REINC_TRY(ensure_side_streams(ctx));
    REINC_TRY(ensure_local(ctx, L, s));
    ctx->scratch_reset();
    const Params p = split_params(c, params);
    const int64_t n = c.num_nodes;
    const int Lg = c.num_gcn_layers, H = c.rnn_hidden;
    const int lstm = c.rnn_kind == REINC_RNN_LSTM;
    const float *nof = nullptr;
    // The GCN part of a timestep does not depend on the recurrent state; with overlap enabled it runs ahead on a
    // side stream while the caller's stream steps the recurrent cell (the cell of snapshot t beside the GCN layers
    // of t+1).  By default both share the caller's stream.
    hipStream_t g = ctx->overlap ? ctx->side[0] : s;
    REINC_TRY(order_after(ctx, s, g));
    for (int32_t i = 0; i < L; ++i) {
        const int32_t t = t0 + i;
        REINC_TRY(ensure_layer1(ctx, t, g));
        const Snapshot &sn = ctx->snaps[t];
        LocalStep &st = ctx->local[i];
        gemm_rows(ctx, g, (const void *)ctx->gcache[t], 0, n, c.dims[0], c.dims[1], (const float *)sn.q, p.W[1], 0, c.dims[1],
                  p.b[1], 1, nof, nof, st.H[1]);
        for (int l = 2; l <= Lg; ++l) {
            aggregate_full(ctx, sn.row_ptr, sn.col, sn.long_rows, sn.n_long_rows, st.H[l - 1], 0, c.dims[l - 1], c.self_loop,
                           sn.p, nullptr, nullptr, st.S[l], g);
            gemm_rows(ctx, g, (const void *)st.S[l], 0, n, c.dims[l - 1], c.dims[l], (const float *)sn.q, p.W[l], 0,
                      c.dims[l], p.b[l], 1, nof, nof, st.H[l]);
        }
        REINC_TRY(order_after(ctx, g, s));
        const LocalStep *pv = i ? &ctx->local[i - 1] : nullptr;
        rnn_fused(ctx, s, lstm, (const float *)st.H[Lg], n, c.dims[Lg], H, pv ? (const float *)pv->h : nof,
                  pv ? (const float *)pv->c : nof, p.W_i, p.W_h, p.b_i, p.b_h, st.h, st.c, st.saved);
    }
    const LocalStep &last = ctx->local[L - 1];
    if (target) launch_mse(last.h, target, n * H, ctx->loss_partial, loss_out, s);
    if (h_last) REINC_HIP(ctx, hipMemcpyAsync(h_last, last.h, uint64_t(n) * H * 4, hipMemcpyDeviceToDevice, s));
    REINC_HIP(ctx, hipGetLastError());
    ctx->local_valid = true;
    ctx->local_t0 = t0;
    return REINC_OK;
}

int reinc_backward_window(reinc_ctx *ctx, int32_t t0, int32_t L, const float *params, const float *target, float *grads,
                          void *stream)
{
    if (!ctx) return REINC_E_ARG;
    REINC_TRY(check_window(ctx, t0, L));
    if (!params || !target || !grads) return ctx->fail(REINC_E_ARG, "null params, target or grads");
    if (!ctx->local_valid || ctx->local_t0 != t0 || int32_t(ctx->local.size()) < L)
        return ctx->fail(REINC_E_STATE, "backward needs the forward pass of the same window [%d, %d) first", t0, t0 + L);
    const reinc_config &c = ctx->cfg;
    hipStream_t s = as_stream(stream);
    REINC_HIP(ctx, hipSetDevice(c.device));
    REINC_TRY(ensure_side_streams(ctx));
    const Params p = split_params(c, params);
    Params gp = split_params(c, grads);
    const int64_t n = c.num_nodes;
    const int Lg = c.num_gcn_layers, H = c.rnn_hidden;
    const int lstm = c.rnn_kind == REINC_RNN_LSTM;
    const int KH = (lstm ? 4 : 3) * H;
    int maxd = H;
    for (int l = 0; l <= Lg; ++l) maxd = std::max(maxd, c.dims[l]);

    ctx->scratch_reset();
    auto f32 = [&](uint64_t count) { return static_cast<float *>(ctx->scratch(count * 4)); };
    float *dh = f32(uint64_t(n) * H), *dh2 = f32(uint64_t(n) * H);
    float *dc = lstm ? f32(uint64_t(n) * H) : nullptr, *dc2 = lstm ? f32(uint64_t(n) * H) : nullptr;
    float *dgi = f32(uint64_t(n) * KH);
    float *dgh = lstm ? dgi : f32(uint64_t(n) * KH);
    float *dz = f32(uint64_t(n) * maxd), *dz2 = f32(uint64_t(n) * maxd), *dagg = f32(uint64_t(n) * maxd);
    // one set of partial slabs per weight matrix: they collect all timesteps and are reduced once at the end
    float *part_wi = static_cast<float *>(ctx->scratch(reduce_partial_bytes(n, c.dims[Lg], KH)));
    float *part_wh = static_cast<float *>(ctx->scratch(reduce_partial_bytes(n, H, KH)));
    float *part_w[REINC_MAX_GCN_LAYERS + 1] = {};
    bool part_ok = part_wi && part_wh;
    for (int l = 1; l <= Lg; ++l) {
        part_w[l] = static_cast<float *>(ctx->scratch(reduce_partial_bytes(n, c.dims[l - 1], c.dims[l])));
        part_ok = part_ok && part_w[l];
    }
    if (!dh || !dh2 || (lstm && (!dc || !dc2)) || !dgi || !dgh || !dz || !dz2 || !dagg || !part_ok) {
        ctx->scratch_reset();
        return ctx->fail(REINC_E_NOMEM, "arena exhausted: no room for the backward scratch buffers");
    }
    float *g = grads;
    launch_fill_f32(g, p.count, 0.0f, s);
    launch_mse_grad(ctx->local[L - 1].h, target, n * H, dh, s);
    const float *dc_in = nullptr;  // zero at the last step
    const float *nof = nullptr;
    // With overlap enabled, per timestep, after the elementwise gate gradients: the caller's stream carries the recurrent chain
    // (gradient w.r.t. h_{t-1}); side 0 and side 1 take the weight-gradient reductions (each weight always on the
    // same stream, so its partial slabs are updated in timestep order); side 2 takes the GCN backward chain.
    hipStream_t s0 = ctx->overlap ? ctx->side[0] : s, s1 = ctx->overlap ? ctx->side[1] : s, s2 = ctx->overlap ? ctx->side[2] : s;
    for (int32_t i = L - 1; i >= 0; --i) {
        const int32_t t = t0 + i;
        const Snapshot &sn = ctx->snaps[t];
        const LocalStep &st = ctx->local[i];
        const LocalStep *pv = i ? &ctx->local[i - 1] : nullptr;
        rnn_backward_elem(ctx, s, lstm, n, H, (const float *)dh, dc_in, (const float *)st.saved,
                          pv ? (const float *)pv->h : nof, pv ? (const float *)pv->c : nof, (const float *)st.c, dgi, dgh, dh2,
                          dc2);
        REINC_TRY(order_after(ctx, s, s0));
        REINC_TRY(order_after(ctx, s, s1));
        REINC_TRY(order_after(ctx, s, s2));
        const float *x = st.H[Lg];
        const int dl = c.dims[Lg];
        const int later = i != L - 1;
        gemm_reduce(ctx, s0, x, dl, nof, (const float *)dgi, KH, n, dl, KH, part_wi, later);
        gemm_reduce(ctx, s1, pv ? (const float *)pv->h : (const float *)ctx->zero_state, H, nof, (const float *)dgh, KH, n, H, KH,
                    part_wh, later);
        // gradient w.r.t. the last GCN layer's pre-activation
        gemm_rows(ctx, s2, (const void *)dgi, 0, n, KH, dl, nof, p.W_i, 1, KH, nof, 0, nof, x, dz);
        if (i > 0) {  // gradient w.r.t. h_{t-1}
            gemm_rows(ctx, s, (const void *)dgh, 0, n, KH, H, nof, p.W_h, 1, KH, nof, 0, lstm ? nof : (const float *)dh2, nof,
                      dh);
            if (lstm) {
                std::swap(dc, dc2);  // dc now holds the gradient w.r.t. c_{t-1}
                dc_in = dc;
                // dc2 is free again; rnn_backward_elem writes the next dc_prev there
            }
        }
        hipStream_t reader_dz2 = nullptr;  // side stream that may still read the buffer behind dz2
        for (int l = Lg; l >= 1; --l) {
            const float *S = l == 1 ? ctx->gcache[t] : st.S[l];
            hipStream_t sr = (l & 1) ? s1 : s0;  // the reduction of layer l always runs on the same side stream
            REINC_TRY(order_after(ctx, s2, sr));
            gemm_reduce(ctx, sr, S, c.dims[l - 1], (const float *)sn.q, (const float *)dz, c.dims[l], n, c.dims[l - 1],
                        c.dims[l], part_w[l], later);
            if (l > 1) {
                gemm_rows(ctx, s2, (const void *)dz, 0, n, c.dims[l], c.dims[l - 1], nof, p.W[l], 1, c.dims[l], nof, 0, nof,
                          nof, dagg);
                if (reader_dz2) REINC_TRY(order_after(ctx, reader_dz2, s2));
                aggregate_full(ctx, sn.col_ptr, sn.row, sn.long_cols, sn.n_long_cols, dagg, 0, c.dims[l - 1], c.self_loop, sn.q,
                               sn.p, st.H[l - 1], dz2, s2);
                std::swap(dz, dz2);
                reader_dz2 = sr;  // this layer's reduction reads what is now dz2
            }
        }
        // the next timestep overwrites the gate gradients and the layer scratch: everything joins first
        REINC_TRY(order_after(ctx, s0, s));
        REINC_TRY(order_after(ctx, s1, s));
        REINC_TRY(order_after(ctx, s2, s));
    }
    launch_reduce_partials(part_wi, n, c.dims[Lg], KH, const_cast<float *>(gp.W_i), const_cast<float *>(gp.b_i), s);
    launch_reduce_partials(part_wh, n, H, KH, const_cast<float *>(gp.W_h), const_cast<float *>(gp.b_h), s);
    for (int l = 1; l <= Lg; ++l)
        launch_reduce_partials(part_w[l], n, c.dims[l - 1], c.dims[l], const_cast<float *>(gp.W[l]),
                               const_cast<float *>(gp.b[l]), s);
    REINC_HIP(ctx, hipGetLastError());
    return REINC_OK;
}

int reinc_cache_clear(reinc_ctx *ctx)
{
    if (!ctx) return REINC_E_ARG;
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
        const uint64_t slot = (uint64_t(ctx->cfg.num_nodes) * ctx->cfg.dims[0] * 4 + 255) & ~uint64_t(255);
        uint64_t count = 0;
        for (float *p : ctx->gcache) count += p != nullptr;
        if (lowest + count * slot == ctx->bottom) ctx->bottom = lowest;
    }
    std::fill(ctx->gcache.begin(), ctx->gcache.end(), nullptr);
    ctx->local_valid = false;
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
