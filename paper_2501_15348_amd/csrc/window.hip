// placeholder
#include "ctx.h"
extern "C" {
int reinc_gcn_transform(reinc_ctx *ctx, const void *, int, int64_t, int32_t, int32_t, const float *, const float *, const float *, int, float *, void *) { return ctx ? ctx->fail(REINC_E_UNSUPPORTED, "not built yet") : REINC_E_ARG; }
int reinc_rnn_step(reinc_ctx *ctx, int, const float *, int64_t, int32_t, int32_t, const float *, const float *, const float *, const float *, const float *, const float *, float *, float *, float *, void *) { return ctx ? ctx->fail(REINC_E_UNSUPPORTED, "not built yet") : REINC_E_ARG; }
int reinc_forward_window(reinc_ctx *ctx, int32_t, int32_t, const float *, const float *, float *, float *, void *) { return ctx ? ctx->fail(REINC_E_UNSUPPORTED, "not built yet") : REINC_E_ARG; }
int reinc_backward_window(reinc_ctx *ctx, int32_t, int32_t, const float *, const float *, float *, void *) { return ctx ? ctx->fail(REINC_E_UNSUPPORTED, "not built yet") : REINC_E_ARG; }
int reinc_cache_clear(reinc_ctx *ctx) { return ctx ? REINC_OK : REINC_E_ARG; }
int reinc_cache_peek(reinc_ctx *ctx, int32_t, const float **o) { if (o) *o = nullptr; return ctx ? REINC_OK : REINC_E_ARG; }
}
