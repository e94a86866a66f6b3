// Neighbourhood aggregation kernels (paper Section 3.2).
//
//   aggregate_rows / aggregate_long_rows : Eq. 1, from scratch.  One wavefront per output row; the
//       wave loads 64 column indices at a time with one coalesced read and hands them round with
//       lane shuffles; a row of d values is read by LPR = d*sizeof(elem)/16 lanes as one 16-byte
//       load each, so 64/LPR source rows are in flight per load instruction and U of those
//       instructions are issued back to back.  Rows with more than kLongRow entries are skipped
//       and taken by a 4-wave block with an LDS reduction (power-law hubs).
//   aggregate_rows_grouped / incremental_rows_grouped : the same sums with one row per group of LPR lanes, for
//       rows of at most kLongRow entries (the bulk of a power-law graph): more independent chains per wave.
//   incremental_rows : Eq. 2 in the form  S_t[r] = S_{t-1}[r] + sum_ins Y_{t-1}[u] - sum_del Y_{t-1}[u]
//       + sum_changed dY[u]  over the rows of R_t only, same lane layout, signed tagged entries.
//
// No atomics anywhere: every output row has one writer and a fixed summation order, so results are
// bit-reproducible from run to run.
#include <algorithm>

#include "ctx.h"

namespace reinc {

namespace {

constexpr int kWavesPerBlock = 4;
constexpr int kUnroll = 8;        // source rows in flight per lane in the wave-per-row kernels
constexpr int kUnrollGrouped = 8;  // in the group-per-row kernels (16 lowers occupancy and measured slower)

template <bool BF16>
struct Row;

template <>
struct Row<false> {
    static constexpr int kVec = 4;
    __device__ static inline void load(const void *base, int64_t row, int d, int li, float (&r)[4])
    {
        const float4 v = *reinterpret_cast<const float4 *>(static_cast<const float *>(base) + row * d + li * 4);
        r[0] = v.x;
        r[1] = v.y;
        r[2] = v.z;
        r[3] = v.w;
    }
};

template <>
struct Row<true> {
    static constexpr int kVec = 8;
    __device__ static inline void load(const void *base, int64_t row, int d, int li, float (&r)[8])
    {
        const uint4 v = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(base) + row * d + li * 8);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            r[2 * i] = __uint_as_float(w[i] << 16);
            r[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
};

template <int VEC>
__device__ inline void load_f32(const float *base, int64_t row, int d, int li, float (&r)[VEC])
{
#pragma unroll
    for (int i = 0; i < VEC; i += 4) {
        const float4 v = *reinterpret_cast<const float4 *>(base + row * d + li * VEC + i);
        r[i] = v.x;
        r[i + 1] = v.y;
        r[i + 2] = v.z;
        r[i + 3] = v.w;
    }
}

template <int VEC>
__device__ inline void store_f32(float *base, int64_t row, int d, int li, const float (&r)[VEC])
{
#pragma unroll
    for (int i = 0; i < VEC; i += 4)
        *reinterpret_cast<float4 *>(base + row * d + li * VEC + i) = make_float4(r[i], r[i + 1], r[i + 2], r[i + 3]);
}

// Sums in_scale[u] * X[u] over the entries [beg, end) handled by this wave (entry e goes to lane group e % G).
template <int LPR, bool BF16>
__device__ inline void gather_segment(const int32_t *idx, int64_t beg, int64_t end, int64_t stride, const void *X,
                                      const float *in_scale, int d, int lane, float (&acc)[Row<BF16>::kVec])
{
    constexpr int VEC = Row<BF16>::kVec;
    constexpr int G = 64 / LPR;
    const int g = lane / LPR, li = lane % LPR;
    for (int64_t base = beg; base < end; base += stride) {
        const int cnt = int(min(int64_t(64), end - base));
        int32_t my_u = 0;
        float my_sc = 1.0f;
        if (lane < cnt) {
            my_u = idx[base + lane];
            if (in_scale) my_sc = in_scale[my_u];
        }
        for (int k = 0; k < cnt; k += G * kUnroll) {
            float r[kUnroll][VEC];
            float sc[kUnroll];
            // the row gathers depend only on the column ids: issue them before touching the gathered scales
#pragma unroll
            for (int j = 0; j < kUnroll; ++j) {
                const int e = k + j * G + g;
                const int32_t u = __shfl(my_u, e & 63);
                if (e < cnt) {
                    Row<BF16>::load(X, u, d, li, r[j]);
                } else {
#pragma unroll
                    for (int i = 0; i < VEC; ++i) r[j][i] = 0.0f;
                }
            }
#pragma unroll
            for (int j = 0; j < kUnroll; ++j) {
                const int e = k + j * G + g;
                sc[j] = __shfl(my_sc, e & 63);
                if (e >= cnt) sc[j] = 0.0f;
            }
#pragma unroll
            for (int j = 0; j < kUnroll; ++j)
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] += sc[j] * r[j][i];
        }
    }
}

template <int LPR, int VEC>
__device__ inline void reduce_groups(float (&acc)[VEC])
{
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] += __shfl_xor(acc[i], off);
}

template <int LPR, bool BF16>
__global__ void __launch_bounds__(64 * kWavesPerBlock)
aggregate_rows(const int64_t *__restrict__ ptr, const int32_t *__restrict__ idx, const void *__restrict__ X, int64_t n,
               int self_loop, const float *__restrict__ in_scale, const float *__restrict__ out_scale,
               const float *__restrict__ mask, float *__restrict__ out, int skip_long)
{
    constexpr int VEC = Row<BF16>::kVec;
    constexpr int D = LPR * VEC;
    const int lane = threadIdx.x & 63;
    const int64_t v = int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
    if (v >= n) return;
    const int64_t beg = ptr[v], end = ptr[v + 1];
    if (skip_long && end - beg > kLongRow) return;
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;
    gather_segment<LPR, BF16>(idx, beg, end, 64, X, in_scale, D, lane, acc);
    reduce_groups<LPR, VEC>(acc);
    if (lane < LPR) {
        if (self_loop) {
            float r[VEC];
            Row<BF16>::load(X, v, D, lane, r);
            const float sc = in_scale ? in_scale[v] : 1.0f;
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] += sc * r[i];
        }
        if (out_scale) {
            const float q = out_scale[v];
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] *= q;
        }
        if (mask) {
            float m[VEC];
            load_f32<VEC>(mask, v, D, lane, m);
#pragma unroll
            for (int i = 0; i < VEC; ++i)
                if (!(m[i] > 0.0f)) acc[i] = 0.0f;
        }
        store_f32<VEC>(out, v, D, lane, acc);
    }
}

// Short rows: every group of LPR lanes owns one output row, so a wave keeps 64/LPR independent
// row-pointer -> column-id -> source-row chains in flight and writes with all 64 lanes.  Rows longer than
// kLongRow are left to the block path.
template <int LPR, bool BF16>
__global__ void __launch_bounds__(64 * kWavesPerBlock)
aggregate_rows_grouped(AggBatch batch, int64_t n, int self_loop)
{
    constexpr int VEC = Row<BF16>::kVec;
    constexpr int D = LPR * VEC;
    constexpr int G = 64 / LPR;
    // blockIdx.y picks the snapshot of the batch: its graph, its input and its output
    const AggItem &it = batch.item[blockIdx.y];
    const int64_t *__restrict__ ptr = it.ptr;
    const int32_t *__restrict__ idx = it.idx;
    const void *__restrict__ X = it.X;
    const float *__restrict__ in_scale = it.in_scale;
    const float *__restrict__ out_scale = it.out_scale;
    const float *__restrict__ mask = it.mask;
    float *__restrict__ out = it.out;
    const int skip_long = it.n_long > 0;
    const int lane = threadIdx.x & 63;
    const int g = lane / LPR, li = lane % LPR, gbase = g * LPR;
    const int64_t v = (int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6)) * G + g;
    const bool live = v < n;
    int64_t beg = 0, end = 0;
    if (live) {
        beg = ptr[v];
        end = ptr[v + 1];
    }
    bool skipped = false;
    if (skip_long && end - beg > kLongRow) {
        skipped = true;
        end = beg;
    }
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;
    // wave-uniform trip counts: the longest row of the wave decides
    int len = int(end - beg);
    int maxlen = len;
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) maxlen = max(maxlen, __shfl_xor(maxlen, off));
    for (int base = 0; base < maxlen; base += LPR) {
        const int cnt = min(LPR, max(len - base, 0));
        int32_t my_u = 0;
        float my_sc = 1.0f;
        if (li < cnt) {
            my_u = idx[beg + base + li];
            if (in_scale) my_sc = in_scale[my_u];
        }
        const int cmax = min(LPR, maxlen - base);
        for (int k = 0; k < cmax; k += kUnrollGrouped) {
            float r[kUnrollGrouped][VEC];
            float sc[kUnrollGrouped];
#pragma unroll
            for (int j = 0; j < kUnrollGrouped; ++j) {
                const int e = k + j;
                const int32_t u = __shfl(my_u, gbase + (e & (LPR - 1)));
                if (e < cnt) {
                    Row<BF16>::load(X, u, D, li, r[j]);
                } else {
#pragma unroll
                    for (int i = 0; i < VEC; ++i) r[j][i] = 0.0f;
                }
            }
#pragma unroll
            for (int j = 0; j < kUnrollGrouped; ++j) {
                const int e = k + j;
                sc[j] = __shfl(my_sc, gbase + (e & (LPR - 1)));
                if (e >= cnt) sc[j] = 0.0f;
            }
#pragma unroll
            for (int j = 0; j < kUnrollGrouped; ++j)
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] += sc[j] * r[j][i];
        }
    }
    if (live && !skipped) {
        if (self_loop) {
            float r[VEC];
            Row<BF16>::load(X, v, D, li, r);
            const float sc = in_scale ? in_scale[v] : 1.0f;
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] += sc * r[i];
        }
        if (out_scale) {
            const float q = out_scale[v];
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] *= q;
        }
        if (mask) {
            float m[VEC];
            load_f32<VEC>(mask, v, D, li, m);
#pragma unroll
            for (int i = 0; i < VEC; ++i)
                if (!(m[i] > 0.0f)) acc[i] = 0.0f;
        }
        store_f32<VEC>(out, v, D, li, acc);
    }
}

// one block of kWavesPerBlock waves per long row; wave w takes the 64-entry chunks w, w+4, ...
template <int LPR, bool BF16>
__global__ void __launch_bounds__(64 * kWavesPerBlock)
aggregate_long_rows(AggBatch batch, int self_loop)
{
    constexpr int VEC = Row<BF16>::kVec;
    constexpr int D = LPR * VEC;
    __shared__ float part[kWavesPerBlock][D];
    const AggItem &it = batch.item[blockIdx.y];
    if (int(blockIdx.x) >= it.n_long) return;  // the grid is as wide as the batch's longest list
    const int64_t *__restrict__ ptr = it.ptr;
    const int32_t *__restrict__ idx = it.idx;
    const void *__restrict__ X = it.X;
    const float *__restrict__ in_scale = it.in_scale;
    const float *__restrict__ out_scale = it.out_scale;
    const float *__restrict__ mask = it.mask;
    float *__restrict__ out = it.out;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t v = it.long_rows[blockIdx.x];
    const int64_t beg = ptr[v], end = ptr[v + 1];
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;
    gather_segment<LPR, BF16>(idx, beg + 64 * w, end, 64 * kWavesPerBlock, X, in_scale, D, lane, acc);
    reduce_groups<LPR, VEC>(acc);
    if (lane < LPR)
#pragma unroll
        for (int i = 0; i < VEC; ++i) part[w][lane * VEC + i] = acc[i];
    __syncthreads();
    if (w == 0 && lane < LPR) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            float s = part[0][lane * VEC + i];
            for (int k = 1; k < kWavesPerBlock; ++k) s += part[k][lane * VEC + i];
            acc[i] = s;
        }
        if (self_loop) {
            float r[VEC];
            Row<BF16>::load(X, v, D, lane, r);
            const float sc = in_scale ? in_scale[v] : 1.0f;
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] += sc * r[i];
        }
        if (out_scale) {
            const float q = out_scale[v];
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] *= q;
        }
        if (mask) {
            float m[VEC];
            load_f32<VEC>(mask, v, D, lane, m);
#pragma unroll
            for (int i = 0; i < VEC; ++i)
                if (!(m[i] > 0.0f)) acc[i] = 0.0f;
        }
        store_f32<VEC>(out, v, D, lane, acc);
    }
}

template <int LPR, bool BF16>
__global__ void __launch_bounds__(64 * kWavesPerBlock)
incremental_rows(const int32_t *__restrict__ rows, int64_t n_rows, const int64_t *__restrict__ ent_ptr,
                 const uint32_t *__restrict__ ent, const void *__restrict__ x_prev, const float *__restrict__ p_prev,
                 const float *__restrict__ dY, const float *S_prev, float *S_out, const float *__restrict__ q,
                 float *__restrict__ agg_out)
{
    constexpr int VEC = Row<BF16>::kVec;
    constexpr int D = LPR * VEC;
    constexpr int G = 64 / LPR;
    const int lane = threadIdx.x & 63;
    const int g = lane / LPR, li = lane % LPR;
    const int64_t w = int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
    if (w >= n_rows) return;
    const int64_t v = rows[w];
    const int64_t beg = ent_ptr[v], end = ent_ptr[v + 1];
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;
    for (int64_t base = beg; base < end; base += 64) {
        const int cnt = int(min(int64_t(64), end - base));
        uint32_t my_e = 0;
        float my_sc = 0.0f;
        if (lane < cnt) {
            my_e = ent[base + lane];
            const uint32_t kind = my_e >> kKindShift;
            if (kind == 2u) {
                my_sc = 1.0f;
            } else {
                my_sc = p_prev ? p_prev[my_e & kPayloadMask] : 1.0f;
                if (kind == 1u) my_sc = -my_sc;
            }
        }
        for (int k = 0; k < cnt; k += G * kUnroll) {
            float r[kUnroll][VEC];
            float sc[kUnroll];
#pragma unroll
            for (int j = 0; j < kUnroll; ++j) {
                const int e = k + j * G + g;
                const uint32_t en = __shfl(my_e, e & 63);
                sc[j] = __shfl(my_sc, e & 63);
                if (e < cnt) {
                    const int64_t u = en & kPayloadMask;
                    if ((en >> kKindShift) == 2u)
                        load_f32<VEC>(dY, u, D, li, r[j]);
                    else
                        Row<BF16>::load(x_prev, u, D, li, r[j]);
                } else {
                    sc[j] = 0.0f;
#pragma unroll
                    for (int i = 0; i < VEC; ++i) r[j][i] = 0.0f;
                }
            }
#pragma unroll
            for (int j = 0; j < kUnroll; ++j)
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] += sc[j] * r[j][i];
        }
    }
    reduce_groups<LPR, VEC>(acc);
    if (lane < LPR) {
        float s[VEC];
        load_f32<VEC>(S_prev, v, D, lane, s);
#pragma unroll
        for (int i = 0; i < VEC; ++i) s[i] += acc[i];
        store_f32<VEC>(S_out, v, D, lane, s);
        if (agg_out) {
            const float qq = q ? q[v] : 1.0f;
#pragma unroll
            for (int i = 0; i < VEC; ++i) s[i] *= qq;
            store_f32<VEC>(agg_out, v, D, lane, s);
        }
    }
}

// Changed rows with at most kLongRow entries, one row per group of LPR lanes (see aggregate_rows_grouped).
template <int LPR, bool BF16>
__global__ void __launch_bounds__(64 * kWavesPerBlock)
incremental_rows_grouped(const int32_t *__restrict__ rows, int64_t n_rows, const int64_t *__restrict__ ent_ptr,
                         const uint32_t *__restrict__ ent, const void *__restrict__ x_prev,
                         const float *__restrict__ p_prev, const float *__restrict__ dY, const float *S_prev, float *S_out,
                         const float *__restrict__ q, float *__restrict__ agg_out)
{
    constexpr int VEC = Row<BF16>::kVec;
    constexpr int D = LPR * VEC;
    constexpr int G = 64 / LPR;
    const int lane = threadIdx.x & 63;
    const int g = lane / LPR, li = lane % LPR, gbase = g * LPR;
    const int64_t w = (int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6)) * G + g;
    const bool live = w < n_rows;
    int64_t v = 0, beg = 0, end = 0;
    if (live) {
        v = rows ? rows[w] : w;  // no row list: every row, so that rows without entries are copied through
        beg = ent_ptr[v];
        end = ent_ptr[v + 1];
    }
    const bool mine = live && end - beg <= kLongRow;  // longer rows belong to the wave-per-row pass
    if (!mine) end = beg;
    float s_old[VEC];
    if (mine) load_f32<VEC>(S_prev, v, D, li, s_old);  // issued early: independent of the entry chain
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;
    const int len = int(end - beg);
    int maxlen = len;
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) maxlen = max(maxlen, __shfl_xor(maxlen, off));
    for (int base = 0; base < maxlen; base += LPR) {
        const int cnt = min(LPR, max(len - base, 0));
        uint32_t my_e = 0;
        float my_sc = 0.0f;
        if (li < cnt) {
            my_e = ent[beg + base + li];
            const uint32_t kind = my_e >> kKindShift;
            if (kind == 2u) {
                my_sc = 1.0f;
            } else {
                my_sc = p_prev ? p_prev[my_e & kPayloadMask] : 1.0f;
                if (kind == 1u) my_sc = -my_sc;
            }
        }
        const int cmax = min(LPR, maxlen - base);
        for (int k = 0; k < cmax; k += kUnrollGrouped) {
            float r[kUnrollGrouped][VEC];
            float sc[kUnrollGrouped];
#pragma unroll
            for (int j = 0; j < kUnrollGrouped; ++j) {
                const int e = k + j;
                const uint32_t en = __shfl(my_e, gbase + (e & (LPR - 1)));
                if (e < cnt) {
                    const int64_t u = en & kPayloadMask;
                    if ((en >> kKindShift) == 2u)
                        load_f32<VEC>(dY, u, D, li, r[j]);
                    else
                        Row<BF16>::load(x_prev, u, D, li, r[j]);
                } else {
#pragma unroll
                    for (int i = 0; i < VEC; ++i) r[j][i] = 0.0f;
                }
            }
#pragma unroll
            for (int j = 0; j < kUnrollGrouped; ++j) {
                const int e = k + j;
                sc[j] = __shfl(my_sc, gbase + (e & (LPR - 1)));
                if (e >= cnt) sc[j] = 0.0f;
            }
#pragma unroll
            for (int j = 0; j < kUnrollGrouped; ++j)
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] += sc[j] * r[j][i];
        }
    }
    if (mine) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) s_old[i] += acc[i];
        store_f32<VEC>(S_out, v, D, li, s_old);
        if (agg_out) {
            const float qq = q ? q[v] : 1.0f;
#pragma unroll
            for (int i = 0; i < VEC; ++i) s_old[i] *= qq;
            store_f32<VEC>(agg_out, v, D, li, s_old);
        }
    }
}

inline int lanes_per_row(int32_t d, int bf16)
{
    int64_t bytes = int64_t(d) * (bf16 ? 2 : 4);
    if (bytes < 16 || bytes > 1024 || (bytes & (bytes - 1))) return 0;
    return int(bytes / 16);
}

template <bool BF16>
void aggregate_dispatch(int lpr, const AggBatch &batch, int64_t n, int self_loop, hipStream_t s, hipEvent_t ev_start,
                        hipEvent_t ev_stop)
{
    const dim3 th(64 * kWavesPerBlock);
#define REINC_AGG_CASE(L)                                                                                          \
    case L: {                                                                                                      \
        const int64_t rows_per_block = int64_t(kWavesPerBlock) * (64 / L);                                         \
        const unsigned blocks = unsigned((n + rows_per_block - 1) / rows_per_block);                               \
        hipExtLaunchKernelGGL((aggregate_rows_grouped<L, BF16>), dim3(blocks, unsigned(batch.count)), th, 0, s,    \
                              ev_start, ev_stop, 0, batch, n, self_loop);                                          \
        break;                                                                                                     \
    }
    switch (lpr) {
        REINC_AGG_CASE(1)
        REINC_AGG_CASE(2)
        REINC_AGG_CASE(4)
        REINC_AGG_CASE(8)
        REINC_AGG_CASE(16)
        REINC_AGG_CASE(32)
        REINC_AGG_CASE(64)
    }
#undef REINC_AGG_CASE
}

template <bool BF16>
void aggregate_long_dispatch(int lpr, const AggBatch &batch, int32_t max_long, int self_loop, hipStream_t s)
{
    const dim3 th(64 * kWavesPerBlock);
    const dim3 grid(unsigned(max_long), unsigned(batch.count));
#define REINC_AGG_CASE(L)                                                         \
    case L:                                                                       \
        aggregate_long_rows<L, BF16><<<grid, th, 0, s>>>(batch, self_loop);       \
        break;
    switch (lpr) {
        REINC_AGG_CASE(1)
        REINC_AGG_CASE(2)
        REINC_AGG_CASE(4)
        REINC_AGG_CASE(8)
        REINC_AGG_CASE(16)
        REINC_AGG_CASE(32)
        REINC_AGG_CASE(64)
    }
#undef REINC_AGG_CASE
}

template <bool BF16>
void incremental_dispatch(int lpr, const int32_t *rows, int64_t n_rows, const int32_t *long_rows, int64_t n_long,
                          const int64_t *ent_ptr, const uint32_t *ent, const void *x_prev, const float *p_prev,
                          const float *dY, const float *S_prev, float *S_out, const float *q, float *agg_out,
                          hipStream_t s)
{
    const dim3 th(64 * kWavesPerBlock);
    const unsigned long_blocks = unsigned((n_long + kWavesPerBlock - 1) / kWavesPerBlock);
#define REINC_INC_CASE(L)                                                                                           \
    case L: {                                                                                                       \
        const int64_t rows_per_block = int64_t(kWavesPerBlock) * (64 / L);                                          \
        const unsigned blocks = unsigned((n_rows + rows_per_block - 1) / rows_per_block);                           \
        incremental_rows_grouped<L, BF16><<<blocks, th, 0, s>>>(rows, n_rows, ent_ptr, ent, x_prev, p_prev, dY, S_prev, \
                                                                S_out, q, agg_out);                                 \
        if (n_long > 0)                                                                                             \
            incremental_rows<L, BF16><<<long_blocks, th, 0, s>>>(long_rows, n_long, ent_ptr, ent, x_prev, p_prev, dY, \
                                                                 S_prev, S_out, q, agg_out);                        \
        break;                                                                                                      \
    }
    switch (lpr) {
        REINC_INC_CASE(1)
        REINC_INC_CASE(2)
        REINC_INC_CASE(4)
        REINC_INC_CASE(8)
        REINC_INC_CASE(16)
        REINC_INC_CASE(32)
        REINC_INC_CASE(64)
    }
#undef REINC_INC_CASE
}

}  // namespace

bool agg_width_supported(int32_t d, int bf16) { return lanes_per_row(d, bf16) != 0; }

void launch_aggregate_batch(const AggBatch &batch, int bf16, int32_t d, int64_t n, int self_loop, hipStream_t s,
                            hipEvent_t ev_start, hipEvent_t ev_stop)
{
    if (n <= 0 || batch.count <= 0) return;
    const int lpr = lanes_per_row(d, bf16);
    if (bf16)
        aggregate_dispatch<true>(lpr, batch, n, self_loop, s, ev_start, ev_stop);
    else
        aggregate_dispatch<false>(lpr, batch, n, self_loop, s, ev_start, ev_stop);
}

void launch_aggregate_long_batch(const AggBatch &batch, int bf16, int32_t d, int self_loop, hipStream_t s)
{
    int32_t max_long = 0;
    for (int i = 0; i < batch.count; ++i) max_long = std::max(max_long, batch.item[i].n_long);
    if (max_long <= 0) return;
    const int lpr = lanes_per_row(d, bf16);
    if (bf16)
        aggregate_long_dispatch<true>(lpr, batch, max_long, self_loop, s);
    else
        aggregate_long_dispatch<false>(lpr, batch, max_long, self_loop, s);
}

void aggregate_full_batch(reinc_ctx *ctx, const AggBatch &batch, int bf16, int32_t d, int self_loop, hipStream_t s)
{
    {
        // the timing events ride on the launch itself, so they carry the kernel's own begin and end
        ProfScope prof(ctx, REINC_K_AGG_FULL, s, true);
        launch_aggregate_batch(batch, bf16, d, ctx->cfg.num_nodes, self_loop, s, prof.start(), prof.stop());
    }
    launch_aggregate_long_batch(batch, bf16, d, self_loop, s);
}

void aggregate_full(reinc_ctx *ctx, const int64_t *ptr, const int32_t *idx, const int32_t *long_rows, int32_t n_long,
                    const void *X, int bf16, int32_t d, int self_loop, const float *in_scale, const float *out_scale,
                    const float *mask, float *out, hipStream_t s)
{
    AggBatch batch;
    batch.count = 1;
    batch.item[0] = AggItem{ptr, idx, X, in_scale, out_scale, mask, out, long_rows, n_long};
    aggregate_full_batch(ctx, batch, bf16, d, self_loop, s);
}

void launch_incremental(const int32_t *rows, int64_t n_rows, const int32_t *long_rows, int64_t n_long,
                        const int64_t *ent_ptr, const uint32_t *ent, const void *x_prev, int bf16, const float *p_prev,
                        const float *dY, int32_t d, const float *S_prev, float *S_out, const float *q, float *agg_out,
                        hipStream_t s)
{
    if (n_rows <= 0) return;
    const int lpr = lanes_per_row(d, bf16);
    if (bf16)
        incremental_dispatch<true>(lpr, rows, n_rows, long_rows, n_long, ent_ptr, ent, x_prev, p_prev, dY, S_prev, S_out, q,
                                   agg_out, s);
    else
        incremental_dispatch<false>(lpr, rows, n_rows, long_rows, n_long, ent_ptr, ent, x_prev, p_prev, dY, S_prev, S_out, q,
                                    agg_out, s);
}

}  // namespace reinc
