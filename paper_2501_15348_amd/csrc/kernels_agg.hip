// Neighbourhood aggregation kernels (paper Section 3.2).
//
//   aggregate_long_rows : Eq. 1, from scratch, rows with more than kLongRow entries (power-law hubs): a 4-wave
//       block per row with an LDS reduction.  A wave loads 64 column indices at a time with one coalesced
//       read and hands them round with lane shuffles; a row of d values is read by LPR = d*sizeof(elem)/16
//       lanes as one 16-byte load each, so 64/LPR source rows are in flight per load instruction and U of
//       those instructions are issued back to back.
//   aggregate_rows_grouped : the same sums with one row per group of LPR lanes, for rows of at most kLongRow
//       entries (the bulk of a power-law graph): more independent chains per wave.
//   incremental_segmented : Eq. 2 in the form  S_t[r] = S_{t-1}[r] + sum_ins Y_{t-1}[u] - sum_del Y_{t-1}[u]
//       + sum_changed dY[u]  over signed tagged entries, the work of a block of rows split by entries.
//
// No atomics anywhere: every output row has one writer and a fixed summation order, so results are
// bit-reproducible from run to run.
#include <algorithm>

#include "ctx.h"

namespace reinc {

namespace {

constexpr int kWavesPerBlock = 4;
constexpr int kUnroll = 8;         // source rows in flight per lane in the wave-per-row kernels
constexpr int kUnrollGrouped = 8;  // in the group-per-row kernels (16 lowers occupancy and measured slower)
// The sum aggregation of bfloat16 rows keeps eight values per gathered row and lane, twice the registers of fp32 rows:
// four rows in flight leave room for more wavefronts per SIMD, which pays (2.5e6 rows of 512 bytes, 5e7 edges: both
// kernels together 6.92 -> 4.73 ms); on fp32 rows four in flight is 1-4 % slower than eight.
template <bool BF16>
constexpr int kSumUnroll = BF16 ? 4 : 8;

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
        for (int k = 0; k < cnt; k += G * kSumUnroll<BF16>) {
            float r[kSumUnroll<BF16>][VEC];
            float sc[kSumUnroll<BF16>];
            // the row gathers depend only on the column ids: issue them before touching the gathered scales
#pragma unroll
            for (int j = 0; j < kSumUnroll<BF16>; ++j) {
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
            for (int j = 0; j < kSumUnroll<BF16>; ++j) {
                const int e = k + j * G + g;
                sc[j] = __shfl(my_sc, e & 63);
                if (e >= cnt) sc[j] = 0.0f;
            }
#pragma unroll
            for (int j = 0; j < kSumUnroll<BF16>; ++j)
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
    const float *__restrict__ add = it.add;
    float *__restrict__ out = it.out;
    const int skip_long = it.n_long > 0;
    const int lane = threadIdx.x & 63;
    const int g = lane / LPR, li = lane % LPR, gbase = g * LPR;
    const int64_t slot = (int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6)) * G + g;
    const bool live = slot < n;
    // with an order list the groups of a wavefront take rows of (nearly) equal length
    const int64_t v = live && it.order ? int64_t(it.order[slot]) : slot;
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
        for (int k = 0; k < cmax; k += kSumUnroll<BF16>) {
            float r[kSumUnroll<BF16>][VEC];
            float sc[kSumUnroll<BF16>];
#pragma unroll
            for (int j = 0; j < kSumUnroll<BF16>; ++j) {
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
            for (int j = 0; j < kSumUnroll<BF16>; ++j) {
                const int e = k + j;
                sc[j] = __shfl(my_sc, gbase + (e & (LPR - 1)));
                if (e >= cnt) sc[j] = 0.0f;
            }
#pragma unroll
            for (int j = 0; j < kSumUnroll<BF16>; ++j)
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
        if (it.bias) {
            float b[VEC];
            load_f32<VEC>(it.bias, 0, D, li, b);
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] += b[i];
        }
        if (it.relu) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = fmaxf(acc[i], 0.0f);
        }
        if (mask) {
            float m[VEC];
            load_f32<VEC>(mask, v, D, li, m);
#pragma unroll
            for (int i = 0; i < VEC; ++i)
                if (!(m[i] > 0.0f)) acc[i] = 0.0f;
        }
        if (add) {
            float a[VEC];
            load_f32<VEC>(add, v, D, li, a);
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] += a[i];
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
    const float *__restrict__ add = it.add;
    float *__restrict__ out = it.out;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t v = it.long_rows[blockIdx.x];
    if (it.row_limit > 0 && v >= it.row_limit) return;  // (the same for the whole block)
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
        if (it.bias) {
            float b[VEC];
            load_f32<VEC>(it.bias, 0, D, lane, b);
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] += b[i];
        }
        if (it.relu) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = fmaxf(acc[i], 0.0f);
        }
        if (mask) {
            float m[VEC];
            load_f32<VEC>(mask, v, D, lane, m);
#pragma unroll
            for (int i = 0; i < VEC; ++i)
                if (!(m[i] > 0.0f)) acc[i] = 0.0f;
        }
        if (add) {
            float a[VEC];
            load_f32<VEC>(add, v, D, lane, a);
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] += a[i];
        }
        store_f32<VEC>(out, v, D, lane, acc);
    }
}

// Rows of S a block of incremental_segmented works on: as many as make a 16 KB tile of fp32 sums (16 rows of 256
// values, 64 rows of 64).  Measured on 2.5e6 rows of 256 bf16 values with 1e7 entries (four gathers in flight): 4 rows
// 2.23 ms, 8 rows 1.78, 16 rows 1.73, 32 rows 2.46; a small tile lets more blocks share a compute unit while they wait
// in different phases.
constexpr int inc_rows_per_block(int d) { return 4096 / d < 8 ? 8 : (4096 / d > 256 ? 256 : 4096 / d); }

// Eq. 2 in the form  S_t[r] = S_{t-1}[r] + sum_ins Y_{t-1}[u] - sum_del Y_{t-1}[u] + sum_changed dY[u].
//
// A block takes RB consecutive rows -- of the whole matrix (rows == null: a new buffer is written, rows without
// entries are copied through) or of the list R_t (in place) -- whose delta entries are adjacent in `ent`.  The work
// is split by ENTRIES, not by rows: every group of LPR lanes gets an equal share of the block's entries and walks it
// eight gathers at a time, whatever rows they belong to, so that a hub row with a thousand entries and a run of rows
// with one entry each cost the same per entry, and no row pointer -> entry -> source row chain is waited for more
// than once per block.  A row that ends inside a group's share is summed in registers and put into the block's LDS
// tile; a row that a share cuts leaves a partial sum in LDS, and the group in whose share the row begins adds the
// pieces in ascending order (fixed order, no atomics: results are bit-reproducible).  Then all threads stream the
// block's rows: S_out = S_prev + tile, coalesced.
template <int LPR, bool BF16>
__global__ void __launch_bounds__(64 * kWavesPerBlock)
incremental_segmented(const int32_t *__restrict__ rows, const int64_t *__restrict__ ptr, int64_t n_rows,
                      const uint32_t *__restrict__ ent, const void *__restrict__ x_prev, const float *__restrict__ p_prev,
                      const float *__restrict__ dY, const float *S_prev, float *S_out, const float *__restrict__ q,
                      float *__restrict__ agg_out, int copy_unchanged)
{
    constexpr int VEC = Row<BF16>::kVec;
    constexpr int D = LPR * VEC;
    constexpr int G = 64 / LPR;
    constexpr int NG = kWavesPerBlock * G;  // lane groups per block
    constexpr int RB = inc_rows_per_block(D);
    constexpr int kThreads = 64 * kWavesPerBlock;
    // gathers a lane has in flight.  Four: the registers of eight (103 at 512-byte bf16 rows) leave four wavefronts per
    // SIMD, and the kernel gains more from the blocks that then share a compute unit than from deeper gathers
    // (2.5e6 rows, 1e7 entries: 2, 3, 4 in flight 1.73 ms, 6: 1.92, 8: 2.22, 12: 2.77, 16: 3.3)
    constexpr int kU = 4;
    __shared__ __align__(16) float tile[RB * D];      // delta sums of the block's rows
    __shared__ __align__(16) float part[NG * D];      // per group: its piece of a row that began in an earlier share
    __shared__ int32_t part_row[2 * NG];              // [2 g]: the row of that piece; [2 g + 1]: the row that begins in
                                                      // share g and goes on into later ones (block-local, -1: none)
    __shared__ int32_t lptr[RB + 1];                  // entry offsets of the block's rows, relative to the first
    __shared__ int32_t lrow[RB];                      // their row ids
    const int tid = threadIdx.x, lane = tid & 63;
    const int g = lane / LPR, li = lane % LPR, gbase = g * LPR;
    const int gid = (tid >> 6) * G + g;
    const int64_t w0 = int64_t(blockIdx.x) * RB;
    const int nr = int(min(int64_t(RB), n_rows - w0));
    const int64_t e0 = ptr[w0];
    for (int i = tid; i <= nr; i += kThreads) lptr[i] = int32_t(ptr[w0 + i] - e0);
    for (int i = tid; i < nr; i += kThreads) lrow[i] = rows ? rows[w0 + i] : int32_t(w0 + i);
    for (int i = tid; i < 2 * NG; i += kThreads) part_row[i] = -1;
    for (int i = tid; i < nr * D / 4; i += kThreads) reinterpret_cast<float4 *>(tile)[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();
    const int ne = lptr[nr];
    const int share = (ne + NG - 1) / NG;
    const int a = min(gid * share, ne), b = min(a + share, ne);
    if (a < b) {
        // the row that holds entry a: lptr[row] <= a < lptr[row + 1]
        int lo = 0, hi = nr;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (lptr[mid] <= a)
                lo = mid;
            else
                hi = mid;
        }
        int row = lo;
        int row_end = lptr[row + 1];
        bool began_earlier = lptr[row] < a;
        float acc[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;
        auto put = [&](float *dst) {
#pragma unroll
            for (int i = 0; i < VEC; i += 4)
                *reinterpret_cast<float4 *>(dst + li * VEC + i) = make_float4(acc[i], acc[i + 1], acc[i + 2], acc[i + 3]);
        };
        for (int base = a; base < b; base += LPR) {
            const int cnt = min(LPR, b - base);
            uint32_t my_e = 0;
            float my_sc = 0.0f;
            if (li < cnt) {
                my_e = ent[e0 + base + li];
                const uint32_t kind = my_e >> kKindShift;
                if (kind == 2u) {
                    my_sc = 1.0f;
                } else {
                    my_sc = p_prev ? p_prev[my_e & kPayloadMask] : 1.0f;
                    if (kind == 1u) my_sc = -my_sc;
                }
            }
            for (int k = 0; k < cnt; k += kU) {
                float r[kU][VEC];
                float sc[kU];
#pragma unroll
                for (int j = 0; j < kU; ++j) {
                    const int e = k + j;
                    const uint32_t en = __shfl(my_e, gbase + (e & (LPR - 1)));
                    if (e < cnt) {
                        const int64_t u = en & kPayloadMask;
                        if constexpr (!BF16) {
                            // both kinds of source are fp32 rows of the same width: one load from a selected base
                            const float *src = (en >> kKindShift) == 2u ? dY : static_cast<const float *>(x_prev);
                            load_f32<VEC>(src, u, D, li, r[j]);
                        } else if ((en >> kKindShift) == 2u) {
                            load_f32<VEC>(dY, u, D, li, r[j]);
                        } else {
                            Row<BF16>::load(x_prev, u, D, li, r[j]);
                        }
                    }
                }
#pragma unroll
                for (int j = 0; j < kU; ++j) sc[j] = __shfl(my_sc, gbase + ((k + j) & (LPR - 1)));
#pragma unroll
                for (int j = 0; j < kU; ++j) {
                    const int e = k + j;
                    if (e < cnt) {
                        if (base + e >= row_end) {  // the current row ended inside this share
                            if (began_earlier) {
                                put(part + gid * D);
                                if (li == 0) part_row[2 * gid] = row;
                                began_earlier = false;
                            } else {
                                put(tile + row * D);
                            }
#pragma unroll
                            for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;
                            do {
                                ++row;
                                row_end = lptr[row + 1];
                            } while (base + e >= row_end);
                        }
#pragma unroll
                        for (int i = 0; i < VEC; ++i) acc[i] += sc[j] * r[j][i];
                    }
                }
            }
        }
        // the last row of the share
        if (began_earlier) {
            put(part + gid * D);
            if (li == 0) part_row[2 * gid] = row;
        } else {
            put(tile + row * D);  // complete, or the first piece of a row that goes on: only this group writes it
            if (row_end > b && li == 0) part_row[2 * gid + 1] = row;
        }
    }
    __syncthreads();
    {
        // a row cut by share boundaries: the group it began in adds the pieces, in ascending order
        const int r = part_row[2 * gid + 1];
        if (r >= 0) {
            float sum[VEC];
#pragma unroll
            for (int i = 0; i < VEC; ++i) sum[i] = tile[r * D + li * VEC + i];
            for (int g2 = gid + 1; g2 < NG && part_row[2 * g2] == r; ++g2)
#pragma unroll
                for (int i = 0; i < VEC; ++i) sum[i] += part[g2 * D + li * VEC + i];
#pragma unroll
            for (int i = 0; i < VEC; ++i) tile[r * D + li * VEC + i] = sum[i];
        }
    }
    __syncthreads();
    // stream the block's rows: four rows per group in flight
    constexpr int kRowsInFlight = 4;
    for (int i0 = gid; i0 < nr; i0 += kRowsInFlight * NG) {
        float s[kRowsInFlight][VEC];
        bool act[kRowsInFlight], has[kRowsInFlight];
#pragma unroll
        for (int u = 0; u < kRowsInFlight; ++u) {
            const int i = i0 + u * NG;
            has[u] = i < nr && lptr[i + 1] > lptr[i];
            act[u] = i < nr && (copy_unchanged || has[u]);
            if (act[u]) load_f32<VEC>(S_prev, lrow[i], D, li, s[u]);
        }
#pragma unroll
        for (int u = 0; u < kRowsInFlight; ++u) {
            const int i = i0 + u * NG;
            if (!act[u]) continue;
            const int64_t v = lrow[i];
            if (has[u]) {  // (a row without entries is copied as it is: bitwise, -0 included)
#pragma unroll
                for (int k = 0; k < VEC; ++k) s[u][k] += tile[i * D + li * VEC + k];
            }
            store_f32<VEC>(S_out, v, D, li, s[u]);
            if (agg_out && has[u]) {
                const float qq = q ? q[v] : 1.0f;
#pragma unroll
                for (int k = 0; k < VEC; ++k) s[u][k] *= qq;
                store_f32<VEC>(agg_out, v, D, li, s[u]);
            }
        }
    }
}

// ---- max / min aggregators (Section 3.2) ----------------------------------------------------------------
// M[v, j] = max over the sources u of v (and v itself with a self-loop) of X[u, j], C[v, j] = the source that
// attains it (the smallest id among equals), 0 / -1 for a target without any source.  min is computed as the max
// of the negated values (sign = -1; negation is exact), so both share one code path and one tie rule.
// Inside the kernels "no source yet" is (m, c) = (-inf, kNoSource), which makes the update one branch-free
// comparison chain; it is turned into the stored (0, -1) at the end.
constexpr int32_t kNoSource = 0x7fffffff;

__device__ inline void mm_update(float x, int32_t u, float &m, int32_t &c)
{
    const bool better = (x > m) | ((x == m) & (u < c));
    m = better ? x : m;
    c = better ? u : c;
}

template <int VEC>
__device__ inline void mm_store(float *out, int32_t *contrib, int64_t v, int d, int li, float sign, float (&m)[VEC],
                                const int32_t (&c)[VEC])
{
    int32_t cs[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        const bool none = c[i] == kNoSource;
        m[i] = none ? 0.0f : sign * m[i];
        cs[i] = none ? -1 : c[i];
    }
    store_f32<VEC>(out, v, d, li, m);
#pragma unroll
    for (int i = 0; i < VEC; i += 4)
        *reinterpret_cast<int4 *>(contrib + v * d + li * VEC + i) = make_int4(cs[i], cs[i + 1], cs[i + 2], cs[i + 3]);
}

// From scratch, rows of at most kLongRow entries: one row per group of LPR lanes (see aggregate_rows_grouped).
// list == nullptr: rows 0 .. count_host-1; else the listed rows (count_dev, if given, points at their number on the
// device: the rows that the incremental pass handed back).  Longer rows are left to minmax_long_rows.
// The gathers of a trip are unconditional: a position past the end of the row repeats the row's last entry, which
// a maximum does not notice.
template <int LPR, bool BF16>
__global__ void __launch_bounds__(64 * kWavesPerBlock)
minmax_rows_grouped(const int32_t *__restrict__ list, const int32_t *__restrict__ count_dev, int64_t count_host,
                    const int64_t *__restrict__ ptr, const int32_t *__restrict__ idx, const void *__restrict__ X,
                    int self_loop, float sign, float *__restrict__ out, int32_t *__restrict__ contrib)
{
    constexpr int VEC = Row<BF16>::kVec;
    constexpr int D = LPR * VEC;
    constexpr int G = 64 / LPR;
    const int lane = threadIdx.x & 63;
    const int g = lane / LPR, li = lane % LPR, gbase = g * LPR;
    const int64_t w = (int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6)) * G + g;
    const int64_t count = count_dev ? int64_t(*count_dev) : count_host;
    bool live = w < count;
    int64_t v = 0, beg = 0, end = 0;
    if (live) {
        v = list ? list[w] : w;
        beg = ptr[v];
        end = ptr[v + 1];
    }
    if (end - beg > kLongRow) {
        live = false;
        end = beg;
    }
    float m[VEC];
    int32_t c[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        m[i] = -INFINITY;
        c[i] = kNoSource;
    }
    const int len = int(end - beg);
    int maxlen = len;
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) maxlen = max(maxlen, __shfl_xor(maxlen, off));
    for (int base = 0; base < maxlen; base += LPR) {
        const int cnt = min(LPR, max(len - base, 0));
        int32_t my_u = 0;
        if (li < cnt) my_u = idx[beg + base + li];
        const int cmax = min(LPR, maxlen - base);
        const int last = max(cnt - 1, 0);
        for (int k = 0; k < cmax; k += kUnrollGrouped) {
            float r[kUnrollGrouped][VEC];
            int32_t us[kUnrollGrouped];
#pragma unroll
            for (int j = 0; j < kUnrollGrouped; ++j) {
                us[j] = __shfl(my_u, gbase + min(k + j, last));  // (row 0 for a group without entries: ignored below)
                Row<BF16>::load(X, us[j], D, li, r[j]);
            }
            if (cnt > 0) {
#pragma unroll
                for (int j = 0; j < kUnrollGrouped; ++j)
#pragma unroll
                    for (int i = 0; i < VEC; ++i) mm_update(sign * r[j][i], us[j], m[i], c[i]);
            }
        }
    }
    if (live) {
        if (self_loop) {
            float r[VEC];
            Row<BF16>::load(X, v, D, li, r);
#pragma unroll
            for (int i = 0; i < VEC; ++i) mm_update(sign * r[i], int32_t(v), m[i], c[i]);
        }
        mm_store<VEC>(out, contrib, v, D, li, sign, m, c);
    }
}

// From scratch, one block of kWavesPerBlock waves per listed row of any length: the long rows of a snapshot; with
// `flags` (indexed by row id) only those that the incremental pass marked.
// Wave w takes the 64-entry chunks w, w + kWavesPerBlock, ...; groups and waves hold disjoint subsets of the
// sources and are combined at the end (the rule does not depend on the order).
template <int LPR, bool BF16>
__global__ void __launch_bounds__(64 * kWavesPerBlock)
minmax_long_rows(const int32_t *__restrict__ list, const int32_t *__restrict__ flags,
                 const int64_t *__restrict__ ptr, const int32_t *__restrict__ idx, const void *__restrict__ X, int self_loop,
                 float sign, float *__restrict__ out, int32_t *__restrict__ contrib)
{
    constexpr int VEC = Row<BF16>::kVec;
    constexpr int D = LPR * VEC;
    constexpr int G = 64 / LPR;
    __shared__ float pm[kWavesPerBlock][D];
    __shared__ int32_t pc[kWavesPerBlock][D];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int g = lane / LPR, li = lane % LPR;
    const int64_t v = list[blockIdx.x];
    if (flags && !flags[v]) return;  // the incremental pass did not ask for this row
    const int64_t beg = ptr[v], end = ptr[v + 1];
    float m[VEC];
    int32_t c[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        m[i] = -INFINITY;
        c[i] = kNoSource;
    }
    for (int64_t base = beg + 64 * w; base < end; base += 64 * kWavesPerBlock) {
        const int cnt = int(min(int64_t(64), end - base));
        int32_t my_u = 0;
        if (lane < cnt) my_u = idx[base + lane];
        for (int k = 0; k < cnt; k += G * kUnroll) {
            float r[kUnroll][VEC];
            int32_t us[kUnroll];
#pragma unroll
            for (int j = 0; j < kUnroll; ++j) {  // a position past the end repeats the chunk's last entry
                us[j] = __shfl(my_u, min(k + j * G + g, cnt - 1));
                Row<BF16>::load(X, us[j], D, li, r[j]);
            }
#pragma unroll
            for (int j = 0; j < kUnroll; ++j)
#pragma unroll
                for (int i = 0; i < VEC; ++i) mm_update(sign * r[j][i], us[j], m[i], c[i]);
        }
    }
    if (self_loop && w == 0 && g == 0) {
        float r[VEC];
        Row<BF16>::load(X, v, D, li, r);
#pragma unroll
        for (int i = 0; i < VEC; ++i) mm_update(sign * r[i], int32_t(v), m[i], c[i]);
    }
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            const float xm = __shfl_xor(m[i], off);
            const int32_t xc = __shfl_xor(c[i], off);
            mm_update(xm, xc, m[i], c[i]);
        }
    if (lane < LPR)
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            pm[w][lane * VEC + i] = m[i];
            pc[w][lane * VEC + i] = c[i];
        }
    __syncthreads();
    if (w == 0 && lane < LPR) {
#pragma unroll
        for (int k = 1; k < kWavesPerBlock; ++k)
#pragma unroll
            for (int i = 0; i < VEC; ++i) mm_update(pm[k][lane * VEC + i], pc[k][lane * VEC + i], m[i], c[i]);
        mm_store<VEC>(out, contrib, v, D, li, sign, m, c);
    }
}

// Incremental step (the paper's procedure): one changed row per group of LPR lanes.  The row's merged delta entries
// name the sources whose contribution disappeared (deleted edges, changed sources) and those whose value is new
// (inserted edges, changed sources), inserted edges first.  If a disappeared source is still the recorded
// contributor of any feature when it is met (an arriving value that has already replaced it makes the loss
// harmless), the row is aggregated from scratch: by the same lane group right away when the row has at most
// kLongRow sources, else by the block-per-row kernel (the row is marked in `hub_flags`).  Otherwise the old result
// combined with the new values is the answer.  Rows with more than kLongRow delta entries are aggregated from
// scratch without looking.  rows == nullptr: every row of the graph (rows without entries are copied to the new
// buffers).  block_counts[blockIdx.x] receives the block's number of rows aggregated from scratch.
template <int LPR, bool BF16>
__global__ void __launch_bounds__(64 * kWavesPerBlock)
minmax_incremental_grouped(const int32_t *__restrict__ rows, int64_t n_rows, const int64_t *__restrict__ ent_ptr,
                           const uint32_t *__restrict__ ent, const int32_t *__restrict__ changed,
                           const int64_t *__restrict__ ptr, const int32_t *__restrict__ idx, const void *__restrict__ x_cur,
                           int self_loop, float sign, const float *M_prev, const int32_t *C_prev, float *M_out, int32_t *C_out,
                           int32_t *__restrict__ hub_flags, int32_t *__restrict__ block_counts)
{
    constexpr int VEC = Row<BF16>::kVec;
    constexpr int D = LPR * VEC;
    constexpr int G = 64 / LPR;
    __shared__ int blk_redone;
    if (threadIdx.x == 0) blk_redone = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int g = lane / LPR, li = lane % LPR, gbase = g * LPR;
    const int64_t w = (int64_t(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6)) * G + g;
    const bool live = w < n_rows;
    int64_t v = 0, beg = 0, end = 0;
    if (live) {
        v = rows ? rows[w] : w;
        beg = ent_ptr[v];
        end = ent_ptr[v + 1];
    }
    const bool too_long = end - beg > kLongRow;
    if (too_long) end = beg;
    float m[VEC];
    int32_t c[VEC], c0[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        m[i] = -INFINITY;
        c[i] = kNoSource;
    }
    if (live) {
        load_f32<VEC>(M_prev, v, D, li, m);
#pragma unroll
        for (int i = 0; i < VEC; i += 4) {
            const int4 t = *reinterpret_cast<const int4 *>(C_prev + v * D + li * VEC + i);
            c[i] = t.x, c[i + 1] = t.y, c[i + 2] = t.z, c[i + 3] = t.w;
        }
#pragma unroll
        for (int i = 0; i < VEC; ++i) {  // back to the "max of sign * x" form
            m[i] = c[i] < 0 ? -INFINITY : sign * m[i];
            c[i] = c[i] < 0 ? kNoSource : c[i];
        }
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) c0[i] = c[i];  // the contributors recorded before this step
    int hit = 0;
    const int len = int(end - beg);
    int maxlen = len;
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) maxlen = max(maxlen, __shfl_xor(maxlen, off));
    for (int base = 0; base < maxlen; base += LPR) {
        const int cnt = min(LPR, max(len - base, 0));
        int32_t my_u = 0, my_kind = 1;
        if (li < cnt) {
            const uint32_t e = ent[beg + base + li];
            my_kind = int32_t(e >> kKindShift);
            my_u = int32_t(e & kPayloadMask);
            if (my_kind == 2) my_u = changed[my_u];
        }
        const int cmax = min(LPR, maxlen - base);
        const int last = max(cnt - 1, 0);
        for (int k = 0; k < cmax; k += kUnrollGrouped) {
            float r[kUnrollGrouped][VEC];
            int32_t us[kUnrollGrouped], kinds[kUnrollGrouped];
#pragma unroll
            for (int j = 0; j < kUnrollGrouped; ++j) {  // unconditional gathers; a position past the end repeats the last entry
                us[j] = __shfl(my_u, gbase + min(k + j, last));
                kinds[j] = __shfl(my_kind, gbase + min(k + j, last));
                Row<BF16>::load(x_cur, us[j], D, li, r[j]);
            }
            if (cnt > 0) {
#pragma unroll
                for (int j = 0; j < kUnrollGrouped; ++j) {
                    // a deleted edge or a changed source: its old contribution is gone; that matters if it was the
                    // recorded contributor and no arriving value has replaced it yet
                    // (a repeated last entry may bring its value again, but is looked up only once)
                    const bool gone = (kinds[j] != 0) & (k + j < cnt), arrives = kinds[j] != 1;
#pragma unroll
                    for (int i = 0; i < VEC; ++i) {
                        hit |= int(gone & (c0[i] == us[j]) & (c[i] == us[j]));
                        // a deleted edge brings nothing: (-inf, kNoSource) never wins
                        mm_update(arrives ? sign * r[j][i] : -INFINITY, arrives ? us[j] : kNoSource, m[i], c[i]);
                    }
                }
            }
        }
    }
    // any lane of the group may have seen the hit
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) hit |= __shfl_xor(hit, off);
    const bool redo_row = live && (hit || too_long);
    // from scratch, by the same group, when the whole row is short
    int64_t fbeg = 0, fend = 0;
    if (redo_row) {
        fbeg = ptr[v];
        fend = ptr[v + 1];
    }
    const bool hub = fend - fbeg > kLongRow;
    if (hub) fend = fbeg;
    if (redo_row) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            m[i] = -INFINITY;
            c[i] = kNoSource;
        }
    }
    const int flen = int(fend - fbeg);
    int fmax = flen;
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) fmax = max(fmax, __shfl_xor(fmax, off));
    for (int base = 0; base < fmax; base += LPR) {
        const int cnt = min(LPR, max(flen - base, 0));
        int32_t my_u = 0;
        if (li < cnt) my_u = idx[fbeg + base + li];
        const int cmax = min(LPR, fmax - base);
        const int last = max(cnt - 1, 0);
        for (int k = 0; k < cmax; k += kUnrollGrouped) {
            float r[kUnrollGrouped][VEC];
            int32_t us[kUnrollGrouped];
#pragma unroll
            for (int j = 0; j < kUnrollGrouped; ++j) {
                us[j] = __shfl(my_u, gbase + min(k + j, last));
                Row<BF16>::load(x_cur, us[j], D, li, r[j]);
            }
            if (cnt > 0) {
#pragma unroll
                for (int j = 0; j < kUnrollGrouped; ++j)
#pragma unroll
                    for (int i = 0; i < VEC; ++i) mm_update(sign * r[j][i], us[j], m[i], c[i]);
            }
        }
    }
    if (live) {
        if (redo_row && hub) {
            if (li == 0) hub_flags[v] = 1;  // (a plain store: thousands of atomics on one counter would serialise)
        } else {
            if (redo_row && self_loop) {
                float r[VEC];
                Row<BF16>::load(x_cur, v, D, li, r);
#pragma unroll
                for (int i = 0; i < VEC; ++i) mm_update(sign * r[i], int32_t(v), m[i], c[i]);
            }
            if (redo_row || len > 0 || M_out != M_prev) mm_store<VEC>(M_out, C_out, v, D, li, sign, m, c);
        }
        if (redo_row && li == 0) atomicAdd(&blk_redone, 1);
    }
    __syncthreads();
    if (threadIdx.x == 0) block_counts[blockIdx.x] = blk_redone;
}

// work[0] = sum of the per-block counts, in a fixed order
__global__ void __launch_bounds__(256) sum_counts_kernel(const int32_t *__restrict__ counts, int64_t n, int32_t *__restrict__ out)
{
    __shared__ int red[256];
    int t = 0;
    for (int64_t i = threadIdx.x; i < n; i += 256) t += counts[i];
    red[threadIdx.x] = t;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (int(threadIdx.x) < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = red[0];
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
void incremental_dispatch(int lpr, const int32_t *rows, const int64_t *ptr, int64_t n_rows, const uint32_t *ent,
                          const void *x_prev, const float *p_prev, const float *dY, const float *S_prev, float *S_out,
                          const float *q, float *agg_out, int copy_unchanged, hipStream_t s, hipEvent_t ev_start,
                          hipEvent_t ev_stop)
{
    const dim3 th(64 * kWavesPerBlock);
#define REINC_INC_CASE(L)                                                                                              \
    case L: {                                                                                                          \
        constexpr int rb = inc_rows_per_block(L * Row<BF16>::kVec);                                                    \
        const unsigned blocks = unsigned((n_rows + rb - 1) / rb);                                                      \
        hipExtLaunchKernelGGL((incremental_segmented<L, BF16>), dim3(blocks), th, 0, s, ev_start, ev_stop, 0, rows,    \
                              ptr, n_rows, ent, x_prev, p_prev, dY, S_prev, S_out, q, agg_out, copy_unchanged);        \
        break;                                                                                                         \
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

#define REINC_LPR_SWITCH(lpr, CASE) \
    switch (lpr) {                  \
        CASE(1)                     \
        CASE(2)                     \
        CASE(4)                     \
        CASE(8)                     \
        CASE(16)                    \
        CASE(32)                    \
        CASE(64)                    \
    }

template <bool BF16>
void minmax_full_dispatch(int lpr, const int64_t *ptr, const int32_t *idx, const int32_t *long_rows, int32_t n_long,
                          const void *X, int64_t n, int self_loop, float sign, float *out, int32_t *contrib, hipStream_t s)
{
    const dim3 th(64 * kWavesPerBlock);
#define REINC_CASE(L)                                                                                                  \
    case L: {                                                                                                          \
        const int64_t rows_per_block = int64_t(kWavesPerBlock) * (64 / L);                                             \
        const unsigned blocks = unsigned((n + rows_per_block - 1) / rows_per_block);                                   \
        minmax_rows_grouped<L, BF16><<<blocks, th, 0, s>>>(nullptr, nullptr, n, ptr, idx, X, self_loop, sign, out, contrib); \
        if (n_long > 0)                                                                                                \
            minmax_long_rows<L, BF16><<<unsigned(n_long), th, 0, s>>>(long_rows, nullptr, ptr, idx, X, self_loop, sign,    \
                                                                      out, contrib);                                   \
        break;                                                                                                         \
    }
    REINC_LPR_SWITCH(lpr, REINC_CASE)
#undef REINC_CASE
}

template <bool BF16>
void minmax_incremental_dispatch(int lpr, const int32_t *rows, int64_t n_rows, const int32_t *long_rows, int32_t n_long,
                                 const int64_t *ent_ptr, const uint32_t *ent, const int32_t *changed, const int64_t *ptr,
                                 const int32_t *idx, const void *x_cur, int self_loop, float sign, const float *M_prev,
                                 const int32_t *C_prev, float *M_out, int32_t *C_out, int32_t *hub_flags, int32_t *block_counts,
                                 int32_t *stat_out, hipStream_t s)
{
    const dim3 th(64 * kWavesPerBlock);
#define REINC_CASE(L)                                                                                                   \
    case L: {                                                                                                           \
        const int64_t rows_per_block = int64_t(kWavesPerBlock) * (64 / L);                                              \
        const unsigned blocks = unsigned((n_rows + rows_per_block - 1) / rows_per_block);                               \
        minmax_incremental_grouped<L, BF16><<<blocks, th, 0, s>>>(rows, n_rows, ent_ptr, ent, changed, ptr, idx, x_cur, \
                                                                  self_loop, sign, M_prev, C_prev, M_out, C_out,        \
                                                                  hub_flags, block_counts);                             \
        if (n_long > 0)                                                                                                 \
            minmax_long_rows<L, BF16><<<unsigned(n_long), th, 0, s>>>(long_rows, hub_flags, ptr, idx, x_cur, self_loop, \
                                                                      sign, M_out, C_out);                              \
        sum_counts_kernel<<<1, 256, 0, s>>>(block_counts, blocks, stat_out);                                            \
        break;                                                                                                          \
    }
    REINC_LPR_SWITCH(lpr, REINC_CASE)
#undef REINC_CASE
}

}  // namespace

bool agg_width_supported(int32_t d, int bf16) { return lanes_per_row(d, bf16) != 0; }

void launch_aggregate_batch(const AggBatch &batch, int bf16, int32_t d, int64_t n, int self_loop, hipStream_t s,
                            hipEvent_t ev_start, hipEvent_t ev_stop)
{
    if (n <= 0 || batch.count <= 0) return;
    const int lpr = lanes_per_row(d, bf16);
    // Rows by falling length (AggItem::order) keep the lane groups of a wavefront equally busy.  That pays while the
    // gathered matrix stays in the caches and the kernel is bound by what a wavefront has in flight (100 000 rows of
    // 256 bytes: 154 -> 140 us per launch of eight snapshots); on matrices far beyond the caches the kernel is bound
    // by HBM either way and the scattered row pointers and output rows cost 2-5 % (1e6 rows of 512 bytes; 5e5 rows of
    // 256 bytes of a graph whose rows are equally long anyway).
    constexpr uint64_t kOrderedBelowBytes = 64ull << 20;
    AggBatch plain;
    const AggBatch *use = &batch;
    if (uint64_t(n) * uint64_t(d) * (bf16 ? 2 : 4) > kOrderedBelowBytes) {
        plain = batch;
        for (int i = 0; i < plain.count; ++i) plain.item[i].order = nullptr;
        use = &plain;
    }
    if (bf16)
        aggregate_dispatch<true>(lpr, *use, n, self_loop, s, ev_start, ev_stop);
    else
        aggregate_dispatch<false>(lpr, *use, n, self_loop, s, ev_start, ev_stop);
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

void aggregate_full_batch(reinc_ctx *ctx, const AggBatch &batch, int bf16, int32_t d, int self_loop, hipStream_t s, int64_t n_rows)
{
    {
        // the timing events ride on the launch itself, so they carry the kernel's own begin and end
        ProfScope prof(ctx, REINC_K_AGG_FULL, s, true);
        launch_aggregate_batch(batch, bf16, d, n_rows >= 0 ? n_rows : ctx->cfg.num_nodes, self_loop, s, prof.start(), prof.stop());
    }
    launch_aggregate_long_batch(batch, bf16, d, self_loop, s);
}

void aggregate_full(reinc_ctx *ctx, const int64_t *ptr, const int32_t *idx, const int32_t *long_rows, int32_t n_long,
                    const void *X, int bf16, int32_t d, int self_loop, const float *in_scale, const float *out_scale,
                    const float *mask, float *out, hipStream_t s, const int32_t *order)
{
    AggBatch batch;
    batch.count = 1;
    batch.item[0] = AggItem{ptr, idx, X, in_scale, out_scale, mask, nullptr, out, long_rows, n_long};
    batch.item[0].order = order;
    aggregate_full_batch(ctx, batch, bf16, d, self_loop, s);
}

void launch_incremental(const int32_t *rows, const int64_t *row_ent, int64_t n_rows, const int64_t *ent_ptr,
                        const uint32_t *ent, const void *x_prev, int bf16, const float *p_prev, const float *dY, int32_t d,
                        const float *S_prev, float *S_out, const float *q, float *agg_out, hipStream_t s, hipEvent_t ev_start,
                        hipEvent_t ev_stop)
{
    if (n_rows <= 0) return;
    const int lpr = lanes_per_row(d, bf16);
    // listed rows: their entries are adjacent, row_ent holds the offsets by list position; every row: ent_ptr by row id
    const int64_t *ptr = rows ? row_ent : ent_ptr;
    const int copy_unchanged = rows == nullptr;
    if (bf16)
        incremental_dispatch<true>(lpr, rows, ptr, n_rows, ent, x_prev, p_prev, dY, S_prev, S_out, q, agg_out, copy_unchanged, s,
                                   ev_start, ev_stop);
    else
        incremental_dispatch<false>(lpr, rows, ptr, n_rows, ent, x_prev, p_prev, dY, S_prev, S_out, q, agg_out, copy_unchanged, s,
                                    ev_start, ev_stop);
}

void launch_minmax_full(const int64_t *ptr, const int32_t *idx, const int32_t *long_rows, int32_t n_long, const void *X,
                        int bf16, int32_t d, int64_t n, int self_loop, int is_max, float *out, int32_t *contrib, hipStream_t s)
{
    if (n <= 0) return;
    const int lpr = lanes_per_row(d, bf16);
    const float sign = is_max ? 1.0f : -1.0f;
    if (bf16)
        minmax_full_dispatch<true>(lpr, ptr, idx, long_rows, n_long, X, n, self_loop, sign, out, contrib, s);
    else
        minmax_full_dispatch<false>(lpr, ptr, idx, long_rows, n_long, X, n, self_loop, sign, out, contrib, s);
}

void launch_minmax_incremental(const int32_t *rows, int64_t n_rows, const int32_t *long_rows, int32_t n_long,
                               const int64_t *ent_ptr, const uint32_t *ent, const int32_t *changed, const int64_t *ptr,
                               const int32_t *idx, const void *x_cur, int bf16, int32_t d, int self_loop, int is_max,
                               const float *M_prev, const int32_t *C_prev, float *M_out, int32_t *C_out, int32_t *hub_flags,
                               int32_t *block_counts, int32_t *stat_out, hipStream_t s)
{
    if (n_rows <= 0) return;
    const int lpr = lanes_per_row(d, bf16);
    const float sign = is_max ? 1.0f : -1.0f;
    if (bf16)
        minmax_incremental_dispatch<true>(lpr, rows, n_rows, long_rows, n_long, ent_ptr, ent, changed, ptr, idx, x_cur,
                                          self_loop, sign, M_prev, C_prev, M_out, C_out, hub_flags, block_counts, stat_out, s);
    else
        minmax_incremental_dispatch<false>(lpr, rows, n_rows, long_rows, n_long, ent_ptr, ent, changed, ptr, idx, x_cur,
                                           self_loop, sign, M_prev, C_prev, M_out, C_out, hub_flags, block_counts, stat_out, s);
}

}  // namespace reinc
