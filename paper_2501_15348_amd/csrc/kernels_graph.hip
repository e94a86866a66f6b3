// Integer kernels: exclusive scan, change-set flags, and the snapshot-diff builder that turns two
// consecutive canonical CSRs (sorted edge keys) into the insert / delete CSRs and the merged signed delta rows
// (paper Section 3.2: delta graphs of edge deletions and insertions, with a node's feature change
// folded in through its out-edges).  All outputs are unique, so they can be compared bit for bit.
#include <climits>

#include "ctx.h"

#include <algorithm>

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

// X[rows[r]] = vals[r], rows of `chunks` 16-byte pieces
__global__ void length_keys(const int64_t *ptr, int64_t n, uint64_t *keys)
{
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v >= n) return;
    const int64_t len = min(ptr[v + 1] - ptr[v], int64_t(kLongRow + 1));
    keys[v] = (uint64_t(kLongRow + 1 - len) << 32) | uint64_t(v);
}

__global__ void scatter_rows(const uint4 *vals, const int32_t *rows, int64_t nrows, int32_t chunks, uint4 *x)
{
    int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i >= nrows * chunks) return;
    int64_t r = i / chunks;
    x[int64_t(rows[r]) * chunks + (i - r * chunks)] = vals[i];
}

__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float(uint32_t(b) << 16); }

inline unsigned blocks_for(int64_t n, int threads) { return unsigned((n + threads - 1) / threads); }

// ---- the diff builder, for many snapshot pairs in one launch: blockIdx.y picks the pair -------------------------
// Two consecutive snapshots are two CSRs with ascending columns, i.e. two sorted lists of edge keys.  A block takes
// kDiffRows consecutive rows: their entries are one contiguous piece of each column list, which the block loads
// once, coalesced, into LDS (up to kDiffCap entries each; a block whose rows hold more, around a hub, searches
// the lists in global memory instead).  Every entry then looks itself up in the same row of the other snapshot --
// a bisection in LDS: absent entries of t are inserted edges, absent entries of t-1 deleted ones, and an entry of t
// whose source is in the change set is a feature-change entry.  Pass 1 leaves four counts per ROW (inserted, deleted,
// all entries, row changes at all) and one BIT per entry and kind; prefix sums over the N rows give the row pointers
// of the three outputs; pass 2 reads the bits and writes every flagged entry where the row pointers and a running
// count inside the block put it (the outputs are row-major, so positions only grow through a block).
constexpr int kDiffRows = 64;  // (at most 64: one wavefront scans a block's per-row counts)
// 2048 entries of each list keep a block at 17 KB of LDS, so that eight blocks share a compute unit (with 4096: four
// blocks, and pass 1 took 1.5 times as long: it waits on dependent LDS reads)
constexpr int kDiffCap = 2048;
constexpr int kDiffThreads = 256;
constexpr int kDiffItems = 8;  // consecutive entries a thread takes per round of pass 2

// stage 0a: cflags[v] = degree of v changed (SYM only: its normalised features change), else 0
__global__ void steps_init_flags(const DiffStep *steps, int64_t n, int sym)
{
    const DiffStep &st = steps[blockIdx.y];
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v >= n) return;
    // under the symmetric normalisation a node's row of Y changes when its source-side scale does, i.e. when its
    // degree does (the scales are compared, not the row lengths: a node batch extracted from a larger graph carries
    // the scales of that graph, and its rows need not hold all of a node's edges)
    st.cflags[v] = sym && st.p_a && st.p_b ? st.p_a[v] != st.p_b[v]
                                           : (sym && (st.rp_a[v + 1] - st.rp_a[v]) != (st.rp_b[v + 1] - st.rp_b[v]));
}

// stage 0b: rows whose features were re-assigned (delta-mode loading keeps their list) and really differ from the
// row before (the change set is defined by the values, not by the list): one thread per 16-byte piece of a listed row
__global__ void steps_flags_list(const DiffStep *steps, int32_t chunks)
{
    const DiffStep &st = steps[blockIdx.y];
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (!st.feat_rows || i >= st.n_feat_rows * chunks) return;
    const int64_t r = i / chunks;
    const int64_t at = int64_t(st.feat_rows[r]) * chunks + (i - r * chunks);
    const uint4 x = static_cast<const uint4 *>(st.x_a)[at], y = static_cast<const uint4 *>(st.x_b)[at];
    if (x.x != y.x || x.y != y.y || x.z != y.z || x.w != y.w) st.cflags[st.feat_rows[r]] = 1;
}

// stage 1a: the change set as one bit per node (64 nodes per word: small enough to stay in the L2 while every edge
// looks its source up)
__global__ void steps_bits(const DiffStep *steps, int64_t n)
{
    const DiffStep &st = steps[blockIdx.y];
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    const unsigned long long m = __ballot(v < n && st.cflags[v] != 0);
    if ((threadIdx.x & 63) == 0 && v < n) st.bits[v >> 6] = m;
}

__device__ inline bool bit_of(const uint64_t *bits, int64_t u) { return (bits[u >> 6] >> (u & 63)) & 1; }

// the row that holds entry e: off[r] <= e < off[r + 1]  (off ascending, off[0] = 0, e < off[nr])
__device__ inline int row_of(const int32_t *off, int nr, int e)
{
    int lo = 0, hi = nr;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (off[mid] <= e)
            lo = mid;
        else
            hi = mid;
    }
    return lo;
}

// Is `key` in the ascending list col[beg, end)?  The search starts at position `hint` and gallops away from it before
// it bisects: between consecutive snapshots most of a row is unchanged, so an entry sits within a few places of where
// it sits in the other snapshot's row, and one or two probes settle it.
__device__ inline bool sorted_has(const int32_t *col, int beg, int end, int hint, int32_t key)
{
    if (beg >= end) return false;
    int p = min(max(hint, beg), end - 1);
    int32_t c = col[p];
    if (c == key) return true;
    int lo, hi;  // the key, if present, lies in [lo, hi)
    if (c < key) {
        lo = p + 1;
        int step = 1;
        hi = lo;
        while (hi < end && col[hi] < key) {
            lo = hi + 1;
            hi += step;
            step <<= 1;
        }
        hi = min(hi + 1, end);
    } else {
        hi = p;
        int step = 1;
        lo = hi;
        while (lo > beg && col[lo - 1] > key) {
            hi = lo - 1;
            lo -= step;
            step <<= 1;
        }
        lo = max(lo - 1, beg);
    }
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (col[mid] < key)
            lo = mid + 1;
        else
            hi = mid;
    }
    return lo < end && col[lo] == key;
}

// what a block of the diff kernels keeps in LDS
struct DiffTile {
    int32_t offa[kDiffRows + 1], offb[kDiffRows + 1];  // entry offsets of the block's rows, relative to the first
    int32_t la[kDiffCap], lb[kDiffCap];                // the column lists (when both fit)
};

// loads the offsets and, if both pieces fit, the column lists; returns whether they are in LDS
__device__ inline bool diff_load(const DiffStep &st, DiffTile &t, int64_t v0, int nr, int64_t &a0, int64_t &b0, bool lists)
{
    a0 = st.rp_a[v0];
    b0 = st.rp_b[v0];
    for (int i = threadIdx.x; i <= nr; i += kDiffThreads) {
        t.offa[i] = int32_t(st.rp_a[v0 + i] - a0);
        t.offb[i] = int32_t(st.rp_b[v0 + i] - b0);
    }
    __syncthreads();
    const int na = t.offa[nr], nb = t.offb[nr];
    const bool fits = lists && na <= kDiffCap && nb <= kDiffCap;
    if (fits) {
        for (int i = threadIdx.x; i < na; i += kDiffThreads) t.la[i] = st.col_a[a0 + i];
        for (int i = threadIdx.x; i < nb; i += kDiffThreads) t.lb[i] = st.col_b[b0 + i];
    }
    __syncthreads();
    return fits;
}

// Where the flag bits of a block's entries begin, in 64-bit words: one bit per entry of the block's piece of a column
// list, 64 consecutive entries per word.  The pieces of consecutive blocks are adjacent in the list, so
// piece_start / 64 + block index leaves every block room for its last, partly filled word.
__device__ inline int64_t mask_base(int64_t piece_start) { return piece_start / 64 + blockIdx.x; }

// pass 1 over one list: `mine` against `other`.  A wavefront takes 64 consecutive entries at a time, one per lane
// (coalesced, conflict-free reads); absent entries are counted per row in cnt_absent, entries whose source is in the
// change set in cnt_hit (bits == null: not wanted), and both kinds are noted as one bit per entry for pass 2 (a
// wavefront's ballot is the word of its 64 entries).
__device__ inline void diff_count_list(const int32_t *mine, const int32_t *off_mine, const int32_t *other, const int32_t *off_other,
                                       int nr, const uint64_t *bits, int32_t *cnt_absent, int32_t *cnt_hit, uint64_t *mask_absent,
                                       uint64_t *mask_hit)
{
    const int total = off_mine[nr];
    const int lane = threadIdx.x & 63;
    static_assert(kDiffRows <= 64, "a lane holds the first entry of one row");
    const int my_start = lane < nr ? off_mine[lane] : INT_MAX;  // (row `lane` begins here)
    for (int base = int(threadIdx.x >> 6) * 64; base < total; base += kDiffThreads) {
        const int e = base + lane;
        bool absent = false, hit = false;
        // The row of every entry of the window: the row that holds its first entry is a count over the lanes' row
        // starts (the same for all lanes); the rows that begin inside the window are few, and each is handed, as a
        // scalar, to the lanes at or behind its first entry.
        const int r0 = __popcll(__ballot(my_start <= base)) - 1;
        int r = r0;
        for (int k = r0 + 1; k < nr; ++k) {
            const int start = __builtin_amdgcn_readlane(my_start, k);
            if (start > base + 63) break;
            if (e >= start) r = k;
        }
        if (e < total) {
            const int32_t u = mine[e];
            const int ob = off_other[r];
            absent = !sorted_has(other, ob, off_other[r + 1], ob + (e - off_mine[r]), u);
            hit = bits && bit_of(bits, u);
            if (absent) atomicAdd(&cnt_absent[r], 1);
            if (hit) atomicAdd(&cnt_hit[r], 1);
        }
        const unsigned long long m_abs = __ballot(absent), m_hit = __ballot(hit);
        if (lane == 0) {
            mask_absent[base / 64] = m_abs;
            if (mask_hit) mask_hit[base / 64] = m_hit;
        }
    }
}

__global__ void __launch_bounds__(kDiffThreads) diff_count(const DiffStep *steps, int64_t n, int self_loop)
{
    __shared__ DiffTile t;
    __shared__ int32_t cnt[3][kDiffRows];  // inserted, deleted, feature-change entries per row
    const DiffStep st = steps[blockIdx.y];  // (a copy: the pointers stay in registers across the stores below)
    const int64_t v0 = int64_t(blockIdx.x) * kDiffRows;
    const int nr = int(min(int64_t(kDiffRows), n - v0));
    for (int i = threadIdx.x; i < 3 * kDiffRows; i += kDiffThreads) (&cnt[0][0])[i] = 0;
    int64_t a0, b0;
    const bool fits = diff_load(st, t, v0, nr, a0, b0, true);
    const uint64_t *bits = st.coffs[n] > 0 ? st.bits : nullptr;  // (an empty change set needs no look-ups)
    uint64_t *ma = st.mask_del + mask_base(a0), *mb = st.mask_ins + mask_base(b0), *mh = bits ? st.mask_hit + mask_base(b0) : nullptr;
    if (fits) {
        diff_count_list(t.lb, t.offb, t.la, t.offa, nr, bits, cnt[0], cnt[2], mb, mh);
        diff_count_list(t.la, t.offa, t.lb, t.offb, nr, nullptr, cnt[1], nullptr, ma, nullptr);
    } else {
        diff_count_list(st.col_b + b0, t.offb, st.col_a + a0, t.offa, nr, bits, cnt[0], cnt[2], mb, mh);
        diff_count_list(st.col_a + a0, t.offa, st.col_b + b0, t.offb, nr, nullptr, cnt[1], nullptr, ma, nullptr);
    }
    __syncthreads();
    for (int r = threadIdx.x; r < nr; r += kDiffThreads) {
        const int64_t v = v0 + r;
        const int32_t own = self_loop && bits && bit_of(bits, v);  // the row's own entry: self-loop of a changed node
        const int32_t all = cnt[0][r] + cnt[1][r] + cnt[2][r] + own;
        st.cnt_ins[v] = cnt[0][r];
        st.cnt_del[v] = cnt[1][r];
        st.cnt_ent[v] = all;
        st.row_flag[v] = all > 0;
    }
}

// exclusive prefix of one value per thread over the block (256 threads); *total = the block's sum
__device__ inline uint32_t block_prefix_u32(uint32_t v, uint32_t *wave_sums, uint32_t *total)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
    }
    __syncthreads();  // (wave_sums may still be read from the previous call)
    if (lane == 63) wave_sums[w] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int k = 0; k < kDiffThreads / 64; ++k) {
        if (k < w) before += wave_sums[k];
        all += wave_sums[k];
    }
    *total = all;
    return before + incl - v;
}

// pass 2 over one list, by the flag bits of pass 1 (a thread takes the byte of kDiffItems = 8 consecutive entries).
// IS_B: `mine` is snapshot t (absent = inserted, and feature-change entries are written too); else snapshot t-1
// (absent = deleted).  p_ins / p_del / p_ent: the output
// row pointers relative to the block's first row, hit_before: feature-change entries in the block's earlier rows.
template <bool IS_B>
__device__ inline void diff_fill_list(const DiffStep &st, const int32_t *mine, const int32_t *off_mine, int nr,
                                      const uint8_t *mask_absent, const uint8_t *mask_hit, const int32_t *p_ins, const int32_t *p_del,
                                      const int32_t *p_ent, const int32_t *hit_before, int64_t out0, int64_t ent0,
                                      uint32_t *wave_sums)
{
    const int total = off_mine[nr];
    uint32_t run_absent = 0, run_hit = 0;  // entries written by earlier rounds
    for (int base = 0; base < total; base += kDiffThreads * kDiffItems) {
        const int e0 = base + int(threadIdx.x) * kDiffItems;
        uint32_t m_absent = 0, m_hit = 0;
        if (e0 < total) {
            m_absent = mask_absent[e0 / kDiffItems];
            if (IS_B && mask_hit) m_hit = mask_hit[e0 / kDiffItems];
        }
        uint32_t tot;
        const uint32_t ex = block_prefix_u32(uint32_t(__popc(m_absent)) | (uint32_t(__popc(m_hit)) << 16), wave_sums, &tot);
        uint32_t at_absent = run_absent + (ex & 0xFFFFu), at_hit = run_hit + (ex >> 16);
        if (m_absent | m_hit) {
            int r = row_of(off_mine, nr, e0);
#pragma unroll
            for (int j = 0; j < kDiffItems; ++j) {
                if (!((m_absent | m_hit) & (1u << j))) continue;
                const int e = e0 + j;
                while (e >= off_mine[r + 1]) ++r;
                const int32_t u = mine[e];
                if (m_absent & (1u << j)) {
                    if (IS_B) {
                        st.ins_col[out0 + at_absent] = u;
                        st.ent[ent0 + p_ent[r] + (int32_t(at_absent) - p_ins[r])] = uint32_t(u);
                    } else {
                        st.del_col[out0 + at_absent] = u;
                        st.ent[ent0 + p_ent[r] + (p_ins[r + 1] - p_ins[r]) + (int32_t(at_absent) - p_del[r])] =
                            (1u << kKindShift) | uint32_t(u);
                    }
                    ++at_absent;
                }
                if (IS_B && (m_hit & (1u << j))) {
                    st.ent[ent0 + p_ent[r] + (p_ins[r + 1] - p_ins[r]) + (p_del[r + 1] - p_del[r]) + (int32_t(at_hit) - hit_before[r])] =
                        (2u << kKindShift) | uint32_t(st.coffs[u]);
                    ++at_hit;
                }
            }
        }
        run_absent += tot & 0xFFFFu;
        run_hit += tot >> 16;
    }
}

__global__ void __launch_bounds__(kDiffThreads) diff_fill(const DiffStep *steps, int64_t n, int self_loop)
{
    __shared__ int32_t offa[kDiffRows + 1], offb[kDiffRows + 1];
    __shared__ int32_t p_ins[kDiffRows + 1], p_del[kDiffRows + 1], p_ent[kDiffRows + 1], hit_before[kDiffRows + 1];
    __shared__ uint32_t wave_sums[kDiffThreads / 64];
    const DiffStep st = steps[blockIdx.y];  // (a copy: the pointers stay in registers across the stores below)
    const int64_t v0 = int64_t(blockIdx.x) * kDiffRows;
    const int nr = int(min(int64_t(kDiffRows), n - v0));
    const int64_t ins0 = st.ins_ptr[v0], del0 = st.del_ptr[v0], ent0 = st.ent_ptr[v0];
    const int64_t a0 = st.rp_a[v0], b0 = st.rp_b[v0];
    for (int i = threadIdx.x; i <= nr; i += kDiffThreads) {
        offa[i] = int32_t(st.rp_a[v0 + i] - a0);
        offb[i] = int32_t(st.rp_b[v0 + i] - b0);
        p_ins[i] = int32_t(st.ins_ptr[v0 + i] - ins0);
        p_del[i] = int32_t(st.del_ptr[v0 + i] - del0);
        p_ent[i] = int32_t(st.ent_ptr[v0 + i] - ent0);
    }
    __syncthreads();
    const uint64_t *bits = st.coffs[n] > 0 ? st.bits : nullptr;
    static_assert(kDiffRows <= 64, "the prefix sums below take one row per lane");
    if (threadIdx.x < 64) {
        // feature-change entries of the block's earlier rows (a row's entries are its inserted, deleted and
        // feature-change entries and, last, its own): prefix sums over the 64 rows in one wavefront
        const int r = threadIdx.x;
        int32_t mine = 0;
        if (r < nr) {
            const int32_t own = self_loop && bits && bit_of(bits, v0 + r);
            mine = (p_ent[r + 1] - p_ent[r]) - (p_ins[r + 1] - p_ins[r]) - (p_del[r + 1] - p_del[r]) - own;
        }
        int32_t incl = mine;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int32_t up = __shfl_up(incl, off);
            if (r >= off) incl += up;
        }
        if (r <= kDiffRows) hit_before[r] = incl - mine;
        if (kDiffRows == 64 && r == 63) hit_before[64] = incl;
    }
    __syncthreads();
    // only flagged entries are touched, so the column lists are read from global memory (a few scattered words)
    if (p_ins[nr] > 0 || hit_before[nr] > 0)
        diff_fill_list<true>(st, st.col_b + b0, offb, nr, reinterpret_cast<const uint8_t *>(st.mask_ins + mask_base(b0)),
                             bits ? reinterpret_cast<const uint8_t *>(st.mask_hit + mask_base(b0)) : nullptr, p_ins, p_del, p_ent,
                             hit_before, ins0, ent0, wave_sums);
    if (p_del[nr] > 0)
        diff_fill_list<false>(st, st.col_a + a0, offa, nr, reinterpret_cast<const uint8_t *>(st.mask_del + mask_base(a0)), nullptr,
                              p_ins, p_del, p_ent, hit_before, del0, ent0, wave_sums);
    // the rows' own entries and the three lists: changed nodes C_t, changed rows R_t with where their entries begin
    for (int r = threadIdx.x; r < nr; r += kDiffThreads) {
        const int64_t v = v0 + r;
        if (bits && bit_of(bits, v)) {
            const int64_t ci = st.coffs[v];
            st.changed[ci] = int32_t(v);
            if (self_loop) st.ent[ent0 + p_ent[r + 1] - 1] = (2u << kKindShift) | uint32_t(ci);
        }
        if (p_ent[r + 1] > p_ent[r]) {
            const int64_t at = st.roffs[v];
            st.rows[at] = int32_t(v);
            st.row_ent[at] = ent0 + p_ent[r];
        }
        if (v == n - 1) st.row_ent[st.roffs[n]] = st.ent_ptr[n];
    }
}

// stage 2b: dY rows of the changed nodes
__global__ void steps_dy(const DiffStep *steps, int bf16, int32_t d)
{
    const DiffStep &st = steps[blockIdx.y];
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i >= st.n_changed * d) return;
    const int64_t r = i / d;
    const int32_t j = int32_t(i - r * d);
    const int64_t u = st.changed[r];
    float a, b;
    if (bf16) {
        a = bf16_to_f32(static_cast<const uint16_t *>(st.x_a)[u * d + j]);
        b = bf16_to_f32(static_cast<const uint16_t *>(st.x_b)[u * d + j]);
    } else {
        a = static_cast<const float *>(st.x_a)[u * d + j];
        b = static_cast<const float *>(st.x_b)[u * d + j];
    }
    const float pa = st.p_a ? st.p_a[u] : 1.0f, pb = st.p_b ? st.p_b[u] : 1.0f;
    st.dY[i] = pb * b - pa * a;
}

}  // namespace

void launch_diff_stage(int stage, const DiffStep *steps_dev, int count, int64_t n, int64_t max_list, int64_t max_changed, int sym,
                       int self_loop, int bf16, int32_t d, hipStream_t s)
{
    if (count <= 0) return;
    auto grid = [&](int64_t elems) { return dim3(std::max(1u, blocks_for(elems, 256)), unsigned(count)); };
    const dim3 row_blocks(unsigned((n + kDiffRows - 1) / kDiffRows), unsigned(count));
    const int32_t chunks = d * (bf16 ? 2 : 4) / 16;
    switch (stage) {
    case 0:
        steps_init_flags<<<grid(n), 256, 0, s>>>(steps_dev, n, sym);
        if (max_list > 0) steps_flags_list<<<grid(max_list * chunks), 256, 0, s>>>(steps_dev, chunks);
        break;
    case 1:
        steps_bits<<<grid(n), 256, 0, s>>>(steps_dev, n);
        diff_count<<<row_blocks, kDiffThreads, 0, s>>>(steps_dev, n, self_loop);
        break;
    case 2:
        diff_fill<<<row_blocks, kDiffThreads, 0, s>>>(steps_dev, n, self_loop);
        if (max_changed > 0) steps_dy<<<grid(max_changed * d), 256, 0, s>>>(steps_dev, bf16, d);
        break;
    default: break;
    }
}

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

void launch_length_keys(const int64_t *ptr, int64_t n, uint64_t *keys, hipStream_t s)
{
    if (n > 0) length_keys<<<blocks_for(n, 256), 256, 0, s>>>(ptr, n, keys);
}

void launch_long_flags(const int64_t *ptr, int64_t n, int32_t *flag, hipStream_t s)
{
    if (n > 0) long_flags<<<blocks_for(n, 256), 256, 0, s>>>(ptr, n, flag);
}

void launch_scatter_rows(const void *vals, const int32_t *rows, int64_t nrows, int32_t row_bytes, void *x, hipStream_t s)
{
    const int32_t chunks = row_bytes / 16;
    const int64_t total = nrows * chunks;
    if (total > 0)
        scatter_rows<<<blocks_for(total, 256), 256, 0, s>>>(static_cast<const uint4 *>(vals), rows, nrows, chunks,
                                                            static_cast<uint4 *>(x));
}

}  // namespace reinc
