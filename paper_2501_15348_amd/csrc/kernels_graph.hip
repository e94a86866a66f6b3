// Integer kernels: exclusive scan, change-set flags, and the snapshot-diff builder that turns two
// consecutive canonical CSRs (sorted edge keys) into the insert / delete CSRs and the merged signed delta rows
// (paper Section 3.2: delta graphs of edge deletions and insertions, with a node's feature change
// folded in through its out-edges).  All outputs are unique, so they can be compared bit for bit.
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

// ---- the diff builder's stages, for many snapshot pairs in one launch: blockIdx.y picks the pair ----------------
// Each stage kernel does everything of that stage that is independent per element (node or edge); the stages are
// separated by the prefix sums, which turn per-element flags into output positions (so the outputs are ordered and
// duplicate-free without any per-row counting).

// stage 1a: cflags[v] = degree of v changed (SYM only: its normalised features change), else 0
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

// stage 1b: rows whose features were re-assigned (delta-mode loading keeps their list)
__global__ void steps_flags_list(const DiffStep *steps)
{
    const DiffStep &st = steps[blockIdx.y];
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (st.feat_rows && i < st.n_feat_rows) st.cflags[st.feat_rows[i]] = 1;
}

// stage 2: threads [0, na) take the edges of t-1, threads [na, na + nb) those of t
__global__ void steps_edge_flags(const DiffStep *steps)
{
    const DiffStep &st = steps[blockIdx.y];
    int64_t e = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (e < st.na) {
        const int32_t v = st.rowid_a[e], u = st.col_a[e];
        st.absent_a[e] = !row_find(st.col_b, st.rp_b[v], st.rp_b[v + 1], u);
        return;
    }
    e -= st.na;
    if (e >= st.nb) return;
    const int32_t v = st.rowid_b[e], u = st.col_b[e];
    st.absent_b[e] = !row_find(st.col_a, st.rp_a[v], st.rp_a[v + 1], u);
    st.hit_b[e] = st.cflags[u] != 0;
}

// stage 3a: row pointers of the three outputs
__global__ void steps_row_ptrs(const DiffStep *steps, int64_t n, int self_loop)
{
    const DiffStep &st = steps[blockIdx.y];
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v > n) return;
    const int64_t i = st.pos_ins[st.rp_b[v]], d = st.pos_del[st.rp_a[v]];
    st.ins_ptr[v] = i;
    st.del_ptr[v] = d;
    st.ent_ptr[v] = i + d + st.pos_hit[st.rp_b[v]] + (self_loop ? st.coffs[v] : 0);
}

// stage 3b: rows that change at all, rows with many entries
__global__ void steps_row_flags(const DiffStep *steps, int64_t n)
{
    const DiffStep &st = steps[blockIdx.y];
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v >= n) return;
    const int64_t len = st.ent_ptr[v + 1] - st.ent_ptr[v];
    st.row_flag[v] = len > 0;
    st.long_flag[v] = len > kLongRow;
}

// stage 4a: the three lists of nodes (changed nodes with their index, changed rows, long rows)
__global__ void steps_compact(const DiffStep *steps, int64_t n)
{
    const DiffStep &st = steps[blockIdx.y];
    const int64_t v = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (v >= n) return;
    const bool c = st.cflags[v] != 0;
    if (c) st.changed[st.coffs[v]] = int32_t(v);
    st.cindex[v] = c ? int32_t(st.coffs[v]) : -1;
    if (st.row_flag[v]) {
        st.rows[st.roffs[v]] = int32_t(v);
        st.row_ent[st.roffs[v]] = st.ent_ptr[v];
    }
    if (v == n - 1) st.row_ent[st.roffs[n]] = st.ent_ptr[n];
    if (st.long_flag[v]) st.long_rows[st.loffs[v]] = int32_t(v);
}

// stage 4b: dY rows of the changed nodes
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

// stage 4c: the entries.  Threads [0, nb): edges of t (inserted, changed source); [nb, nb + na): edges of t-1
// (deleted); [nb + na, nb + na + n): the rows' own entries (self-loop of a changed node, last in its row).
__global__ void steps_fill(const DiffStep *steps, int64_t n, int self_loop)
{
    const DiffStep &st = steps[blockIdx.y];
    int64_t e = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (e < st.nb) {
        const int32_t v = st.rowid_b[e], u = st.col_b[e];
        if (st.absent_b[e]) {
            const int64_t r = st.pos_ins[e];
            st.ins_col[r] = u;
            st.ent[st.ent_ptr[v] + (r - st.ins_ptr[v])] = uint32_t(u);
        }
        if (st.hit_b[e]) {
            const int64_t base = st.ent_ptr[v] + (st.ins_ptr[v + 1] - st.ins_ptr[v]) + (st.del_ptr[v + 1] - st.del_ptr[v]);
            st.ent[base + (st.pos_hit[e] - st.pos_hit[st.rp_b[v]])] = (2u << kKindShift) | uint32_t(st.cindex[u]);
        }
        return;
    }
    e -= st.nb;
    if (e < st.na) {
        if (!st.absent_a[e]) return;
        const int32_t v = st.rowid_a[e], u = st.col_a[e];
        const int64_t r = st.pos_del[e];
        st.del_col[r] = u;
        st.ent[st.ent_ptr[v] + (st.ins_ptr[v + 1] - st.ins_ptr[v]) + (r - st.del_ptr[v])] = (1u << kKindShift) | uint32_t(u);
        return;
    }
    e -= st.na;
    if (!self_loop || e >= n) return;
    const int32_t ci = st.cindex[e];
    if (ci >= 0) st.ent[st.ent_ptr[e + 1] - 1] = (2u << kKindShift) | uint32_t(ci);
}

}  // namespace

void launch_diff_stage(int stage, const DiffStep *steps_dev, int count, int64_t n, int64_t max_a, int64_t max_b, int64_t max_list,
                       int64_t max_changed, int sym, int self_loop, int bf16, int32_t d, hipStream_t s)
{
    if (count <= 0) return;
    auto grid = [&](int64_t elems) { return dim3(std::max(1u, blocks_for(elems, 256)), unsigned(count)); };
    switch (stage) {
    case 0:
        steps_init_flags<<<grid(n), 256, 0, s>>>(steps_dev, n, sym);
        if (max_list > 0) steps_flags_list<<<grid(max_list), 256, 0, s>>>(steps_dev);
        break;
    case 1: steps_edge_flags<<<grid(max_a + max_b), 256, 0, s>>>(steps_dev); break;
    case 2:
        steps_row_ptrs<<<grid(n + 1), 256, 0, s>>>(steps_dev, n, self_loop);
        steps_row_flags<<<grid(n), 256, 0, s>>>(steps_dev, n);
        break;
    case 3:
        steps_compact<<<grid(n), 256, 0, s>>>(steps_dev, n);
        if (max_changed > 0) steps_dy<<<grid(max_changed * d), 256, 0, s>>>(steps_dev, bf16, d);
        steps_fill<<<grid(max_a + max_b + n), 256, 0, s>>>(steps_dev, n, self_loop);
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
