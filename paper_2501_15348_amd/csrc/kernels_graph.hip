// Integer kernels: exclusive scan, change-set flags, and the snapshot-diff builder that turns two
// consecutive canonical CSRs into the insert / delete CSRs and the merged signed delta rows
// (paper Section 3.2: delta graphs of edge deletions and insertions, with a node's feature change
// folded in through its out-edges).  All outputs are unique, so they can be compared bit for bit.
#include "ctx.h"

namespace reinc {

namespace {

constexpr int kScanThreads = 256;
constexpr int kScanItems = 8;
constexpr int kScanTile = kScanThreads * kScanItems;

__global__ void fill_i32(int32_t *p, int64_t n, int32_t v)
{
    int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i < n) p[i] = v;
}

// block-wide exclusive scan of one value per thread (256 threads); returns the exclusive prefix and the block total
__device__ inline int64_t block_exclusive_scan(int64_t v, int64_t *lds, int64_t *total)
{
    int t = threadIdx.x;
    lds[t] = v;
    __syncthreads();
    for (int off = 1; off < kScanThreads; off <<= 1) {
        int64_t add = t >= off ? lds[t - off] : 0;
        __syncthreads();
        lds[t] += add;
        __syncthreads();
    }
    int64_t incl = lds[t];
    *total = lds[kScanThreads - 1];
    __syncthreads();
    return incl - v;
}

__global__ void __launch_bounds__(kScanThreads) scan_tile_sums(const int32_t *counts, int64_t n, int64_t *tile_sums)
{
    __shared__ int64_t lds[kScanThreads];
    int64_t base = int64_t(blockIdx.x) * kScanTile + int64_t(threadIdx.x) * kScanItems;
    int64_t s = 0;
    for (int k = 0; k < kScanItems; ++k)
        if (base + k < n) s += counts[base + k];
    int64_t total;
    block_exclusive_scan(s, lds, &total);
    if (threadIdx.x == 0) tile_sums[blockIdx.x] = total;
}

// one block: exclusive scan of the tile sums in place
__global__ void __launch_bounds__(kScanThreads) scan_tile_offsets(int64_t *tile_sums, int64_t ntiles)
{
    __shared__ int64_t lds[kScanThreads];
    int64_t running = 0;
    for (int64_t base = 0; base < ntiles; base += kScanThreads) {
        int64_t i = base + threadIdx.x;
        int64_t v = i < ntiles ? tile_sums[i] : 0;
        int64_t total;
        int64_t ex = block_exclusive_scan(v, lds, &total);
        if (i < ntiles) tile_sums[i] = running + ex;
        running += total;
    }
}

__global__ void __launch_bounds__(kScanThreads)
scan_finish(const int32_t *counts, int64_t n, const int64_t *tile_offsets, int64_t *offsets)
{
    __shared__ int64_t lds[kScanThreads];
    int64_t base = int64_t(blockIdx.x) * kScanTile + int64_t(threadIdx.x) * kScanItems;
    int32_t c[kScanItems];
    int64_t s = 0;
    for (int k = 0; k < kScanItems; ++k) {
        c[k] = base + k < n ? counts[base + k] : 0;
        s += c[k];
    }
    int64_t total;
    int64_t ex = block_exclusive_scan(s, lds, &total) + tile_offsets[blockIdx.x];
    for (int k = 0; k < kScanItems; ++k) {
        if (base + k < n) offsets[base + k] = ex;
        ex += c[k];
        if (base + k == n - 1) offsets[n] = ex;
    }
}

__global__ void write_zero_i64(int64_t *p) { p[0] = 0; }

// ---- change-set flags ------------------------------------------------------------------------------------
__global__ void flags_compare(const uint4 *a, const uint4 *b, int64_t nchunks, int32_t chunks_per_row, int32_t *flags)
{
    int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i >= nchunks) return;
    uint4 x = a[i], y = b[i];
    if (x.x != y.x || x.y != y.y || x.z != y.z || x.w != y.w) flags[i / chunks_per_row] = 1;
}

__global__ void flags_list(const int32_t *rows, int64_t nrows, int32_t *flags)
{
    int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i < nrows) flags[rows[i]] = 1;
}

__global__ void flags_degree(const int64_t *rp_a, const int64_t *rp_b, int64_t n, int32_t *flags)
{
    int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v < n && (rp_a[v + 1] - rp_a[v]) != (rp_b[v + 1] - rp_b[v])) flags[v] = 1;
}

// list[offsets[i]] = i for flagged i; index_of[i] = offsets[i] or -1
__global__ void compact(const int32_t *flags, const int64_t *offsets, int64_t n, int32_t *list, int32_t *index_of)
{
    int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i >= n) return;
    bool f = flags[i] != 0;
    if (f) list[offsets[i]] = int32_t(i);
    if (index_of) index_of[i] = f ? int32_t(offsets[i]) : -1;
}

// ---- snapshot diff: a group of kGroup lanes walks one row ------------------------------------------------
constexpr int kGroup = 16;
constexpr int kDiffThreads = 256;
constexpr int kRowsPerBlock = kDiffThreads / kGroup;

__device__ inline bool row_find(const int32_t *col, int64_t beg, int64_t end, int32_t key)
{
    int64_t lo = beg, hi = end;
    while (lo < hi) {
        int64_t mid = (lo + hi) >> 1;
        if (col[mid] < key)
            lo = mid + 1;
        else
            hi = mid;
    }
    return lo < end && col[lo] == key;
}

// Membership of this lane's two values in the other list of a row that fits one group (both lists <= kGroup
// long): the group's lanes hand their values round with shuffles, so no dependent global reads are needed.
// A lane without a value passes -1, which never matches a node id.
__device__ inline void group_membership(int32_t av, int32_t bv, int lane, bool &a_in_b, bool &b_in_a)
{
    const int gbase = lane & ~(kGroup - 1);
    a_in_b = false;
    b_in_a = false;
#pragma unroll
    for (int j = 0; j < kGroup; ++j) {
        const int32_t bj = __shfl(bv, gbase + j);
        const int32_t aj = __shfl(av, gbase + j);
        a_in_b |= (bj == av);
        b_in_a |= (aj == bv);
    }
}

__device__ inline int wave_max(int v)
{
    for (int off = 32; off > 0; off >>= 1) v = max(v, __shfl_xor(v, off));
    return v;
}

// A = snapshot t-1, B = snapshot t.  Per row: |B \ A|, |A \ B|, and the size of the merged delta row.
__global__ void __launch_bounds__(kDiffThreads)
delta_count(const int64_t *rp_a, const int32_t *col_a, const int64_t *rp_b, const int32_t *col_b, const int32_t *cflags,
            int self_loop, int64_t n, int32_t *cnt_ins, int32_t *cnt_del, int32_t *cnt_all, int32_t *row_flag)
{
    const int lane = threadIdx.x & 63;
    const int g = lane / kGroup, li = lane % kGroup;
    const uint64_t gmask = ((uint64_t(1) << kGroup) - 1) << (g * kGroup);
    int64_t v = int64_t(blockIdx.x) * kRowsPerBlock + threadIdx.x / kGroup;
    bool live = v < n;
    int64_t a0 = 0, a1 = 0, b0 = 0, b1 = 0;
    if (live) {
        a0 = rp_a[v];
        a1 = rp_a[v + 1];
        b0 = rp_b[v];
        b1 = rp_b[v + 1];
    }
    int la = int(a1 - a0), lb = int(b1 - b0);
    int iters = (wave_max(max(la, lb)) + kGroup - 1) / kGroup;
    int n_ins = 0, n_del = 0, n_f = 0;
    const bool short_row = la <= kGroup && lb <= kGroup;
    for (int it = 0; it < iters; ++it) {
        int k = it * kGroup + li;
        const int32_t av = k < la ? col_a[a0 + k] : -1;
        const int32_t bv = k < lb ? col_b[b0 + k] : -1;
        bool a_in_b, b_in_a;
        group_membership(av, bv, lane, a_in_b, b_in_a);
        if (!short_row) {
            a_in_b = k < la && row_find(col_b, b0, b1, av);
            b_in_a = k < lb && row_find(col_a, a0, a1, bv);
        }
        const bool is_del = k < la && !a_in_b;
        const bool is_ins = k < lb && !b_in_a;
        const bool is_f = k < lb && cflags[bv] != 0;
        n_del += __popcll(__ballot(is_del) & gmask);
        n_ins += __popcll(__ballot(is_ins) & gmask);
        n_f += __popcll(__ballot(is_f) & gmask);
    }
    if (live && li == 0) {
        if (self_loop && cflags[v]) n_f += 1;
        cnt_ins[v] = n_ins;
        cnt_del[v] = n_del;
        int all = n_ins + n_del + n_f;
        cnt_all[v] = all;
        row_flag[v] = all > 0;
    }
}

__global__ void __launch_bounds__(kDiffThreads)
delta_fill(const int64_t *rp_a, const int32_t *col_a, const int64_t *rp_b, const int32_t *col_b, const int32_t *cindex,
           int self_loop, int64_t n, const int64_t *ins_ptr, int32_t *ins_col, const int64_t *del_ptr, int32_t *del_col,
           const int64_t *ent_ptr, uint32_t *ent)
{
    const int lane = threadIdx.x & 63;
    const int g = lane / kGroup, li = lane % kGroup;
    const uint64_t gmask = ((uint64_t(1) << kGroup) - 1) << (g * kGroup);
    const uint64_t below = (uint64_t(1) << lane) - 1;
    int64_t v = int64_t(blockIdx.x) * kRowsPerBlock + threadIdx.x / kGroup;
    bool live = v < n;
    int64_t a0 = 0, a1 = 0, b0 = 0, b1 = 0, o_ins = 0, o_del = 0, e_ins = 0, e_del = 0, e_f = 0;
    if (live) {
        a0 = rp_a[v];
        a1 = rp_a[v + 1];
        b0 = rp_b[v];
        b1 = rp_b[v + 1];
        o_ins = ins_ptr[v];
        o_del = del_ptr[v];
        e_ins = ent_ptr[v];
        e_del = e_ins + (ins_ptr[v + 1] - o_ins);
        e_f = e_del + (del_ptr[v + 1] - o_del);
    }
    int la = int(a1 - a0), lb = int(b1 - b0);
    int iters = (wave_max(max(la, lb)) + kGroup - 1) / kGroup;
    const bool short_row = la <= kGroup && lb <= kGroup;
    for (int it = 0; it < iters; ++it) {
        int k = it * kGroup + li;
        const int32_t ua = k < la ? col_a[a0 + k] : -1;
        const int32_t ub = k < lb ? col_b[b0 + k] : -1;
        bool a_in_b, b_in_a;
        group_membership(ua, ub, lane, a_in_b, b_in_a);
        if (!short_row) {
            a_in_b = k < la && row_find(col_b, b0, b1, ua);
            b_in_a = k < lb && row_find(col_a, a0, a1, ub);
        }
        const bool is_del = k < la && !a_in_b;
        const bool is_ins = k < lb && !b_in_a;
        const int32_t ci = k < lb ? cindex[ub] : -1;
        const bool is_f = ci >= 0;
        uint64_t m_del = __ballot(is_del) & gmask, m_ins = __ballot(is_ins) & gmask, m_f = __ballot(is_f) & gmask;
        if (is_del) {
            int r = __popcll(m_del & below);
            del_col[o_del + r] = ua;
            ent[e_del + r] = (1u << kKindShift) | uint32_t(ua);
        }
        if (is_ins) {
            int r = __popcll(m_ins & below);
            ins_col[o_ins + r] = ub;
            ent[e_ins + r] = uint32_t(ub);
        }
        if (is_f) {
            int r = __popcll(m_f & below);
            ent[e_f + r] = (2u << kKindShift) | uint32_t(ci);
        }
        int c_del = __popcll(m_del), c_ins = __popcll(m_ins), c_f = __popcll(m_f);
        o_del += c_del;
        e_del += c_del;
        o_ins += c_ins;
        e_ins += c_ins;
        e_f += c_f;
    }
    if (live && li == 0 && self_loop) {
        int ci = cindex[v];
        if (ci >= 0) ent[e_f] = (2u << kKindShift) | uint32_t(ci);
    }
}

// X[rows[r]] = vals[r], rows of `chunks` 16-byte pieces
__global__ void scatter_rows(const uint4 *vals, const int32_t *rows, int64_t nrows, int32_t chunks, uint4 *x)
{
    int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i >= nrows * chunks) return;
    int64_t r = i / chunks;
    x[int64_t(rows[r]) * chunks + (i - r * chunks)] = vals[i];
}

__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float(uint32_t(b) << 16); }

// dY[i] = p_cur[u] X_cur[u] - p_prev[u] X_prev[u],  u = changed[i]
__global__ void dy_rows(const void *x_prev, const void *x_cur, int bf16, const float *p_prev, const float *p_cur,
                        const int32_t *changed, int64_t n_changed, int32_t d, float *dY)
{
    int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i >= n_changed * d) return;
    int64_t r = i / d;
    int32_t j = int32_t(i - r * d);
    int64_t u = changed[r];
    float a, b;
    if (bf16) {
        a = bf16_to_f32(static_cast<const uint16_t *>(x_prev)[u * d + j]);
        b = bf16_to_f32(static_cast<const uint16_t *>(x_cur)[u * d + j]);
    } else {
        a = static_cast<const float *>(x_prev)[u * d + j];
        b = static_cast<const float *>(x_cur)[u * d + j];
    }
    float pa = p_prev ? p_prev[u] : 1.0f, pb = p_cur ? p_cur[u] : 1.0f;
    dY[i] = pb * b - pa * a;
}

inline unsigned blocks_for(int64_t n, int threads) { return unsigned((n + threads - 1) / threads); }

}  // namespace

uint64_t scan_tmp_bytes(int64_t n)
{
    int64_t tiles = (n + kScanTile - 1) / kScanTile;
    return uint64_t(tiles > 0 ? tiles : 1) * sizeof(int64_t);
}

void launch_scan(const int32_t *counts, int64_t *offsets, int64_t n, void *tmp, hipStream_t s)
{
    if (n <= 0) {
        write_zero_i64<<<1, 1, 0, s>>>(offsets);
        return;
    }
    int64_t tiles = (n + kScanTile - 1) / kScanTile;
    int64_t *tile_sums = static_cast<int64_t *>(tmp);
    scan_tile_sums<<<unsigned(tiles), kScanThreads, 0, s>>>(counts, n, tile_sums);
    scan_tile_offsets<<<1, kScanThreads, 0, s>>>(tile_sums, tiles);
    scan_finish<<<unsigned(tiles), kScanThreads, 0, s>>>(counts, n, tile_sums, offsets);
}

void launch_fill_i32(int32_t *p, int64_t n, int32_t v, hipStream_t s)
{
    if (n > 0) fill_i32<<<blocks_for(n, 256), 256, 0, s>>>(p, n, v);
}

void launch_feature_flags_compare(const void *x_prev, const void *x_cur, int64_t n, int32_t row_bytes, int32_t *flags,
                                  hipStream_t s)
{
    int32_t cpr = row_bytes / 16;
    int64_t chunks = n * cpr;
    if (chunks > 0)
        flags_compare<<<blocks_for(chunks, 256), 256, 0, s>>>(static_cast<const uint4 *>(x_prev),
                                                               static_cast<const uint4 *>(x_cur), chunks, cpr, flags);
}

void launch_feature_flags_list(const int32_t *rows, int64_t nrows, int64_t n, int32_t *flags, hipStream_t s)
{
    (void)n;
    if (nrows > 0) flags_list<<<blocks_for(nrows, 256), 256, 0, s>>>(rows, nrows, flags);
}

void launch_degree_flags(const int64_t *rp_prev, const int64_t *rp_cur, int64_t n, int32_t *flags, hipStream_t s)
{
    if (n > 0) flags_degree<<<blocks_for(n, 256), 256, 0, s>>>(rp_prev, rp_cur, n, flags);
}

void launch_compact(const int32_t *flags, const int64_t *offsets, int64_t n, int32_t *list, int32_t *index_of,
                    hipStream_t s)
{
    if (n > 0) compact<<<blocks_for(n, 256), 256, 0, s>>>(flags, offsets, n, list, index_of);
}

void launch_delta_count(const int64_t *rp_a, const int32_t *col_a, const int64_t *rp_b, const int32_t *col_b,
                        const int32_t *cflags, int self_loop, int64_t n, int32_t *cnt_ins, int32_t *cnt_del,
                        int32_t *cnt_all, int32_t *row_flag, hipStream_t s)
{
    if (n > 0)
        delta_count<<<blocks_for(n, kRowsPerBlock), kDiffThreads, 0, s>>>(rp_a, col_a, rp_b, col_b, cflags, self_loop, n,
                                                                          cnt_ins, cnt_del, cnt_all, row_flag);
}

void launch_delta_fill(const int64_t *rp_a, const int32_t *col_a, const int64_t *rp_b, const int32_t *col_b,
                       const int32_t *cindex, int self_loop, int64_t n, const int64_t *ins_ptr, int32_t *ins_col,
                       const int64_t *del_ptr, int32_t *del_col, const int64_t *ent_ptr, uint32_t *ent, hipStream_t s)
{
    if (n > 0)
        delta_fill<<<blocks_for(n, kRowsPerBlock), kDiffThreads, 0, s>>>(rp_a, col_a, rp_b, col_b, cindex, self_loop, n,
                                                                         ins_ptr, ins_col, del_ptr, del_col, ent_ptr, ent);
}

void launch_scatter_rows(const void *vals, const int32_t *rows, int64_t nrows, int32_t row_bytes, void *x, hipStream_t s)
{
    const int32_t chunks = row_bytes / 16;
    const int64_t total = nrows * chunks;
    if (total > 0)
        scatter_rows<<<blocks_for(total, 256), 256, 0, s>>>(static_cast<const uint4 *>(vals), rows, nrows, chunks,
                                                            static_cast<uint4 *>(x));
}

void launch_dy(const void *x_prev, const void *x_cur, int bf16, const float *p_prev, const float *p_cur,
               const int32_t *changed, int64_t n_changed, int32_t d, float *dY, hipStream_t s)
{
    int64_t total = n_changed * d;
    if (total > 0)
        dy_rows<<<blocks_for(total, 256), 256, 0, s>>>(x_prev, x_cur, bf16, p_prev, p_cur, changed, n_changed, d, dY);
}

}  // namespace reinc
