// Integer kernels: exclusive scan, change-set flags, and the snapshot-diff builder that turns two
// consecutive canonical CSRs (sorted edge keys) into the insert / delete CSRs and the merged signed delta rows
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

// ---- many scans in one launch ---------------------------------------------------------------------------------
// The tiles of all jobs are numbered consecutively (job j owns tiles [tile0, tile0 + ceil(n / tile))); a block finds
// its job by bisection over tile0.  Same arithmetic as the single scan, so the results are identical.
__device__ inline int find_job(const ScanJob *jobs, int njobs, int64_t tile)
{
    int lo = 0, hi = njobs - 1;  // last job whose tile0 <= tile (jobs without tiles share their successor's tile0 and lose)
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (jobs[mid].tile0 <= tile)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

// a thread's eight consecutive counts: two 16-byte loads where all eight exist and the array is aligned
__device__ inline void load_items(const int32_t *in, int64_t n, int64_t base, int32_t (&c)[kScanItems])
{
    if (base + kScanItems <= n && (reinterpret_cast<uintptr_t>(in) & 15) == 0) {
        const int4 a = *reinterpret_cast<const int4 *>(in + base), b = *reinterpret_cast<const int4 *>(in + base + 4);
        c[0] = a.x, c[1] = a.y, c[2] = a.z, c[3] = a.w, c[4] = b.x, c[5] = b.y, c[6] = b.z, c[7] = b.w;
        return;
    }
    for (int k = 0; k < kScanItems; ++k) c[k] = base + k < n ? in[base + k] : 0;
}

__global__ void __launch_bounds__(kScanThreads) multi_scan_tile_sums(const ScanJob *jobs, int njobs, int64_t *tile_sums)
{
    __shared__ int64_t lds[kScanThreads];
    const ScanJob job = jobs[find_job(jobs, njobs, blockIdx.x)];
    int64_t base = (int64_t(blockIdx.x) - job.tile0) * kScanTile + int64_t(threadIdx.x) * kScanItems;
    int32_t c[kScanItems];
    load_items(job.in, job.n, base, c);
    int64_t s = 0;
    for (int k = 0; k < kScanItems; ++k) s += c[k];
    int64_t total;
    block_exclusive_scan(s, lds, &total);
    if (threadIdx.x == 0) tile_sums[blockIdx.x] = total;
}

// one block per job: exclusive scan of the job's tile sums in place; an empty job gets its single output here
__global__ void __launch_bounds__(kScanThreads) multi_scan_tile_offsets(const ScanJob *jobs, int64_t *tile_sums)
{
    __shared__ int64_t lds[kScanThreads];
    const ScanJob job = jobs[blockIdx.x];
    if (job.n <= 0) {
        if (threadIdx.x == 0) job.out[0] = 0;
        return;
    }
    const int64_t ntiles = (job.n + kScanTile - 1) / kScanTile;
    int64_t *mine = tile_sums + job.tile0;
    int64_t running = 0;
    for (int64_t base = 0; base < ntiles; base += kScanThreads) {
        int64_t i = base + threadIdx.x;
        int64_t v = i < ntiles ? mine[i] : 0;
        int64_t total;
        int64_t ex = block_exclusive_scan(v, lds, &total);
        if (i < ntiles) mine[i] = running + ex;
        running += total;
    }
}

__global__ void __launch_bounds__(kScanThreads) multi_scan_finish(const ScanJob *jobs, int njobs, const int64_t *tile_offsets)
{
    __shared__ int64_t lds[kScanThreads];
    const ScanJob job = jobs[find_job(jobs, njobs, blockIdx.x)];
    int64_t base = (int64_t(blockIdx.x) - job.tile0) * kScanTile + int64_t(threadIdx.x) * kScanItems;
    int32_t c[kScanItems];
    load_items(job.in, job.n, base, c);
    int64_t s = 0;
    for (int k = 0; k < kScanItems; ++k) s += c[k];
    int64_t total;
    int64_t ex = block_exclusive_scan(s, lds, &total) + tile_offsets[blockIdx.x];
    if (base + kScanItems < job.n && (reinterpret_cast<uintptr_t>(job.out) & 15) == 0) {
        // a thread's eight outputs are 64 consecutive bytes: four 16-byte stores
        longlong2 *o = reinterpret_cast<longlong2 *>(job.out + base);
#pragma unroll
        for (int k = 0; k < kScanItems; k += 2) {
            longlong2 v;
            v.x = ex;
            v.y = ex + c[k];
            ex += c[k] + c[k + 1];
            o[k / 2] = v;
        }
        return;
    }
    for (int k = 0; k < kScanItems; ++k) {
        if (base + k < job.n) job.out[base + k] = ex;
        ex += c[k];
        if (base + k == job.n - 1) job.out[job.n] = ex;
    }
}

// dst[i] = *src[i]: the totals of many scans gathered for one copy to the host
__global__ void gather_i64(const int64_t *const *src, int count, int64_t *dst)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) dst[i] = *src[i];
}

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

// ---- canonicalisation of a raw edge list (set semantics) -----------------------------------------------------
// key = target * 2^32 + source; a self-loop or an endpoint outside [0, n) gets the key n * 2^32, which sorts behind
// every valid key and is dropped; an endpoint outside the range also raises the error flag.
__global__ void make_keys(const int32_t *src, const int32_t *dst, int64_t nnz, int64_t n, uint64_t *keys, int32_t *err)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i >= nnz) return;
    const int64_t u = src[i], v = dst[i];
    const bool bad = u < 0 || u >= n || v < 0 || v >= n;
    if (bad) atomicOr(err, 1);
    keys[i] = (bad || u == v) ? (uint64_t(n) << 32) : ((uint64_t(v) << 32) | uint64_t(u));
}

// flag[i] = 1 for the first copy of every valid key of the sorted list
__global__ void unique_flags(const uint64_t *keys, int64_t nnz, int64_t n, int32_t *flag)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i >= nnz) return;
    const uint64_t k = keys[i];
    flag[i] = int64_t(k >> 32) < n && (i == 0 || keys[i - 1] != k);
}

// col[j] = low half, rowid[j] = high half of the j-th kept key; swapped[j] = the key with its halves exchanged
__global__ void scatter_unique(const uint64_t *keys, const int32_t *flag, const int64_t *offs, int64_t nnz, int32_t *col,
                               int32_t *rowid, uint64_t *swapped)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i >= nnz || !flag[i]) return;
    const uint64_t k = keys[i];
    const int64_t j = offs[i];
    col[j] = int32_t(k & 0xFFFFFFFFu);
    rowid[j] = int32_t(k >> 32);
    swapped[j] = (k << 32) | (k >> 32);
}

__global__ void low_halves(const uint64_t *keys, int64_t e, int32_t *out)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i < e) out[i] = int32_t(keys[i] & 0xFFFFFFFFu);
}

// ptr[v] = number of sorted keys whose high half is below v, for v = 0 .. n (binary search per row)
__global__ void ptr_from_sorted(const uint64_t *keys, int64_t e, int64_t n, int64_t *ptr)
{
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v > n) return;
    int64_t lo = 0, hi = e;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (int64_t(keys[mid] >> 32) < v)
            lo = mid + 1;
        else
            hi = mid;
    }
    ptr[v] = lo;
}

__global__ void ptr_from_rowid(const int32_t *rowid, int64_t e, int64_t n, int64_t *ptr)
{
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v > n) return;
    int64_t lo = 0, hi = e;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (rowid[mid] < v)
            lo = mid + 1;
        else
            hi = mid;
    }
    ptr[v] = lo;
}

// q[v] = 1/deg (mean) or deg^-1/2 (sym), deg = self_loop + row length; 0 for deg = 0
__global__ void degree_scales(const int64_t *ptr, int64_t n, int sym, int self_loop, float *q)
{
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v >= n) return;
    const double deg = double(ptr[v + 1] - ptr[v] + self_loop);
    q[v] = deg <= 0.0 ? 0.0f : float(sym ? 1.0 / sqrt(deg) : 1.0 / deg);
}

__global__ void long_flags(const int64_t *ptr, int64_t n, int32_t *flag)
{
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v < n) flag[v] = ptr[v + 1] - ptr[v] > kLongRow;
}

// ---- snapshot diff, one thread per edge -----------------------------------------------------------------
// Every edge of one snapshot looks itself up in the same row of the other snapshot (binary search over that
// row's sorted columns).  Work is per edge, so a hub row costs no more per element than a short one and the
// launch has no long tail; consecutive threads share a row, so the row bounds and the top probes hit in cache.
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

// absent[e] = 1 if edge e of `self` is not in `other`; hit[e] = cflags[col[e]] != 0 (optional)
__global__ void edge_flags(const int32_t *rowid, const int32_t *col, int64_t nnz, const int64_t *other_ptr,
                           const int32_t *other_col, const int32_t *cflags, int32_t *absent, int32_t *hit)
{
    const int64_t e = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (e >= nnz) return;
    const int32_t v = rowid[e], u = col[e];
    absent[e] = !row_find(other_col, other_ptr[v], other_ptr[v + 1], u);
    if (hit) hit[e] = cflags[u] != 0;
}

// Row pointers of the three outputs from the per-edge prefix sums:
//   ins_ptr[v] = pos_ins[rp_b[v]], del_ptr[v] = pos_del[rp_a[v]],
//   ent_ptr[v] = ins_ptr[v] + del_ptr[v] + pos_hit[rp_b[v]] + (self_loop ? pos_self[v] : 0)
__global__ void delta_row_ptrs(const int64_t *rp_a, const int64_t *rp_b, const int64_t *pos_del, const int64_t *pos_ins,
                               const int64_t *pos_hit, const int64_t *pos_self, int self_loop, int64_t n,
                               int64_t *ins_ptr, int64_t *del_ptr, int64_t *ent_ptr)
{
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v > n) return;
    const int64_t i = pos_ins[rp_b[v]], d = pos_del[rp_a[v]];
    ins_ptr[v] = i;
    del_ptr[v] = d;
    ent_ptr[v] = i + d + pos_hit[rp_b[v]] + (self_loop ? pos_self[v] : 0);
}

__global__ void row_nonempty(const int64_t *ent_ptr, int64_t n, int32_t *flag)
{
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v < n) flag[v] = ent_ptr[v + 1] > ent_ptr[v];
}

__global__ void row_long(const int64_t *ent_ptr, int64_t n, int32_t *flag)
{
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v < n) flag[v] = ent_ptr[v + 1] - ent_ptr[v] > kLongRow;
}

// Inserted edges (kind 0) and changed-source entries (kind 2) come from snapshot t's edges.
__global__ void fill_from_cur(const int32_t *rowid, const int32_t *col, int64_t nnz, const int64_t *rp_b,
                              const int32_t *absent, const int32_t *hit, const int64_t *pos_ins, const int64_t *pos_hit,
                              const int32_t *cindex, const int64_t *ins_ptr, const int64_t *del_ptr,
                              const int64_t *ent_ptr, int32_t *ins_col, uint32_t *ent)
{
    const int64_t e = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (e >= nnz) return;
    const int32_t v = rowid[e], u = col[e];
    if (absent[e]) {
        const int64_t r = pos_ins[e];
        ins_col[r] = u;
        ent[ent_ptr[v] + (r - ins_ptr[v])] = uint32_t(u);
    }
    if (hit[e]) {
        const int64_t base = ent_ptr[v] + (ins_ptr[v + 1] - ins_ptr[v]) + (del_ptr[v + 1] - del_ptr[v]);
        ent[base + (pos_hit[e] - pos_hit[rp_b[v]])] = (2u << kKindShift) | uint32_t(cindex[u]);
    }
}

// Deleted edges (kind 1) come from snapshot t-1's edges.
__global__ void fill_from_prev(const int32_t *rowid, const int32_t *col, int64_t nnz, const int32_t *absent,
                               const int64_t *pos_del, const int64_t *ins_ptr, const int64_t *del_ptr,
                               const int64_t *ent_ptr, int32_t *del_col, uint32_t *ent)
{
    const int64_t e = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (e >= nnz || !absent[e]) return;
    const int32_t v = rowid[e], u = col[e];
    const int64_t r = pos_del[e];
    del_col[r] = u;
    ent[ent_ptr[v] + (ins_ptr[v + 1] - ins_ptr[v]) + (r - del_ptr[v])] = (1u << kKindShift) | uint32_t(u);
}

// The row's own entry (self-loop of a changed node) is the last entry of its row.
__global__ void fill_self(const int32_t *cindex, int64_t n, const int64_t *ent_ptr, uint32_t *ent)
{
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v >= n) return;
    const int32_t ci = cindex[v];
    if (ci >= 0) ent[ent_ptr[v + 1] - 1] = (2u << kKindShift) | uint32_t(ci);
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

int64_t scan_tiles(int64_t n) { return n > 0 ? (n + kScanTile - 1) / kScanTile : 0; }

void launch_multi_scan(const ScanJob *jobs_dev, int njobs, int64_t total_tiles, int64_t *tile_sums, hipStream_t s)
{
    if (njobs <= 0) return;
    if (total_tiles > 0) multi_scan_tile_sums<<<unsigned(total_tiles), kScanThreads, 0, s>>>(jobs_dev, njobs, tile_sums);
    multi_scan_tile_offsets<<<unsigned(njobs), kScanThreads, 0, s>>>(jobs_dev, tile_sums);
    if (total_tiles > 0) multi_scan_finish<<<unsigned(total_tiles), kScanThreads, 0, s>>>(jobs_dev, njobs, tile_sums);
}

void launch_gather_i64(const int64_t *const *src_dev, int count, int64_t *dst, hipStream_t s)
{
    if (count > 0) gather_i64<<<(count + 255) / 256, 256, 0, s>>>(src_dev, count, dst);
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

void launch_make_keys(const int32_t *src, const int32_t *dst, int64_t nnz, int64_t n, uint64_t *keys, int32_t *err,
                      hipStream_t s)
{
    if (nnz > 0) make_keys<<<blocks_for(nnz, 256), 256, 0, s>>>(src, dst, nnz, n, keys, err);
}

void launch_unique_flags(const uint64_t *keys, int64_t nnz, int64_t n, int32_t *flag, hipStream_t s)
{
    if (nnz > 0) unique_flags<<<blocks_for(nnz, 256), 256, 0, s>>>(keys, nnz, n, flag);
}

void launch_scatter_unique(const uint64_t *keys, const int32_t *flag, const int64_t *offs, int64_t nnz, int32_t *col,
                           int32_t *rowid, uint64_t *swapped, hipStream_t s)
{
    if (nnz > 0) scatter_unique<<<blocks_for(nnz, 256), 256, 0, s>>>(keys, flag, offs, nnz, col, rowid, swapped);
}

void launch_low_halves(const uint64_t *keys, int64_t e, int32_t *out, hipStream_t s)
{
    if (e > 0) low_halves<<<blocks_for(e, 256), 256, 0, s>>>(keys, e, out);
}

void launch_ptr_from_sorted(const uint64_t *keys, int64_t e, int64_t n, int64_t *ptr, hipStream_t s)
{
    ptr_from_sorted<<<blocks_for(n + 1, 256), 256, 0, s>>>(keys, e, n, ptr);
}

void launch_ptr_from_rowid(const int32_t *rowid, int64_t e, int64_t n, int64_t *ptr, hipStream_t s)
{
    ptr_from_rowid<<<blocks_for(n + 1, 256), 256, 0, s>>>(rowid, e, n, ptr);
}

void launch_degree_scales(const int64_t *ptr, int64_t n, int sym, int self_loop, float *q, hipStream_t s)
{
    if (n > 0) degree_scales<<<blocks_for(n, 256), 256, 0, s>>>(ptr, n, sym, self_loop, q);
}

void launch_long_flags(const int64_t *ptr, int64_t n, int32_t *flag, hipStream_t s)
{
    if (n > 0) long_flags<<<blocks_for(n, 256), 256, 0, s>>>(ptr, n, flag);
}

void launch_edge_flags(const int32_t *rowid, const int32_t *col, int64_t nnz, const int64_t *other_ptr,
                       const int32_t *other_col, const int32_t *cflags, int32_t *absent, int32_t *hit, hipStream_t s)
{
    if (nnz > 0)
        edge_flags<<<blocks_for(nnz, 256), 256, 0, s>>>(rowid, col, nnz, other_ptr, other_col, cflags, absent, hit);
}

void launch_delta_row_ptrs(const int64_t *rp_a, const int64_t *rp_b, const int64_t *pos_del, const int64_t *pos_ins,
                           const int64_t *pos_hit, const int64_t *pos_self, int self_loop, int64_t n, int64_t *ins_ptr,
                           int64_t *del_ptr, int64_t *ent_ptr, int32_t *row_flag, hipStream_t s)
{
    delta_row_ptrs<<<blocks_for(n + 1, 256), 256, 0, s>>>(rp_a, rp_b, pos_del, pos_ins, pos_hit, pos_self, self_loop, n,
                                                          ins_ptr, del_ptr, ent_ptr);
    if (n > 0) row_nonempty<<<blocks_for(n, 256), 256, 0, s>>>(ent_ptr, n, row_flag);
}

void launch_row_long_flags(const int64_t *ent_ptr, int64_t n, int32_t *flag, hipStream_t s)
{
    if (n > 0) row_long<<<blocks_for(n, 256), 256, 0, s>>>(ent_ptr, n, flag);
}

void launch_delta_fill(const int32_t *rowid_a, const int32_t *col_a, int64_t nnz_a, const int32_t *rowid_b,
                       const int32_t *col_b, int64_t nnz_b, const int64_t *rp_b, const int32_t *absent_a,
                       const int32_t *absent_b, const int32_t *hit_b, const int64_t *pos_del, const int64_t *pos_ins,
                       const int64_t *pos_hit, const int32_t *cindex, int self_loop, int64_t n, const int64_t *ins_ptr,
                       int32_t *ins_col, const int64_t *del_ptr, int32_t *del_col, const int64_t *ent_ptr, uint32_t *ent,
                       hipStream_t s)
{
    if (nnz_b > 0)
        fill_from_cur<<<blocks_for(nnz_b, 256), 256, 0, s>>>(rowid_b, col_b, nnz_b, rp_b, absent_b, hit_b, pos_ins, pos_hit,
                                                             cindex, ins_ptr, del_ptr, ent_ptr, ins_col, ent);
    if (nnz_a > 0)
        fill_from_prev<<<blocks_for(nnz_a, 256), 256, 0, s>>>(rowid_a, col_a, nnz_a, absent_a, pos_del, ins_ptr, del_ptr,
                                                              ent_ptr, del_col, ent);
    if (self_loop && n > 0) fill_self<<<blocks_for(n, 256), 256, 0, s>>>(cindex, n, ent_ptr, ent);
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
