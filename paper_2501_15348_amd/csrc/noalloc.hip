// An entry point for callers that cannot allocate device memory or hand over a work buffer: the incremental max / min
// step with its work area in a file-scope device array instead of a caller-provided buffer.
#include "ctx.h"

using namespace reinc;

namespace {

// Work area of reinc_aggregate_incremental_minmax for up to kStaticMaxNodes nodes: 2 N + 4 int32 (the count of
// re-aggregated rows, one mark per row, one count per block).  8 MiB + 256 B per GPU, held until the process ends.
constexpr int64_t kStaticMaxNodes = int64_t(1) << 20;
constexpr int64_t kStaticWords = 2 * kStaticMaxNodes + 64;
static __device__ __align__(256) int32_t scratch[kStaticWords];

// Device address of `scratch` on each GPU (every GPU holds its own copy of the array at its own address); found once
// per device by reinc_create.  Host code uses these pointers, never the array's name.
constexpr int kMaxDevices = 64;
int32_t *scratch_ptr[kMaxDevices] = {};

__global__ void copy_word(const int32_t *src, int32_t *dst)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) *dst = *src;
}

}  // namespace

// Looks up this device's copy of the static work area (the context's device must be current).
int reinc::static_scratch_init(reinc_ctx *ctx)
{
    const int dev = ctx->cfg.device;
    if (dev < 0 || dev >= kMaxDevices) return REINC_OK;  // the static entry point reports it when it is called
    if (scratch_ptr[dev]) return REINC_OK;
    void *p = nullptr;
    REINC_HIP(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return ctx->fail(REINC_E_HIP, "hipGetSymbolAddress returned a null address for the static work area");
    scratch_ptr[dev] = static_cast<int32_t *>(p);
    return REINC_OK;
}

extern "C" int reinc_aggregate_incremental_minmax_static(reinc_ctx *ctx, int32_t t, int op, const float *M_prev,
                                                         const int32_t *C_prev, float *M_out, int32_t *C_out,
                                                         int32_t *n_redone_out, void *stream)
{
    if (!ctx) return REINC_E_ARG;
    if (ctx->N() > kStaticMaxNodes)
        return ctx->fail(REINC_E_ARG, "the static work area serves at most %lld nodes, this context has %lld: use "
                                      "reinc_aggregate_incremental_minmax with a work buffer",
                         (long long)kStaticMaxNodes, (long long)ctx->N());
    const int dev = ctx->cfg.device;
    int32_t *work = dev >= 0 && dev < kMaxDevices ? scratch_ptr[dev] : nullptr;
    if (!work) return ctx->fail(REINC_E_UNSUPPORTED, "no static work area on device %d", dev);
    hipStream_t s = static_cast<hipStream_t>(stream);
    REINC_TRY(reinc::minmax_incremental(ctx, t, op, M_prev, C_prev, M_out, C_out, work, /*timed=*/false, s));
    if (n_redone_out) {
        copy_word<<<1, 64, 0, s>>>(work, n_redone_out);
        REINC_HIP(ctx, hipGetLastError());
    }
    return REINC_OK;
}
