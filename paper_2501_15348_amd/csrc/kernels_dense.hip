// Dense kernels on the fp32 matrix cores (v_mfma_f32_32x32x2_f32, 64-lane wavefronts):
//   gemm_rows    C[n,M] = epilogue( (row_scale .* A)[n,K] * B[K,M] )        GCN update (Section 3.5, Listing 1)
//                                                                          and the input-gradient GEMMs
//   rnn_fused    both gate GEMMs of a GRU / LSTM step plus the gate arithmetic in one pass (Section 3.3:
//                3 gates for GRU, 4 for LSTM)
//   gemm_reduce  C[K,M] = sum over rows of (row_scale .* A)^T G, with the column sums of G: weight and
//                bias gradients; per-chunk partial tiles are summed in a fixed order (no atomics)
//   small elementwise kernels for the recurrent backward step and the loss.
//
// Operand layout of the 32x32x2 instruction: lane l supplies A[l%32][l/32] and B[l/32][l%32]; register r
// of the 16 accumulators holds C[8*(r/4) + 4*(l/32) + r%4][l%32].  The k index is only a summation label,
// so a lane that loads 16 consecutive k values of its row uses element s in step s while the B side
// reads row 16*(l/32)+s of the staged weight chunk: each 128-byte line of A is fetched by one lane pair.
#include "ctx.h"

#include <cstdlib>
#include <type_traits>
#include <cstring>

namespace reinc {

namespace {

typedef float acc16 __attribute__((ext_vector_type(16)));

constexpr int kBK = 32;  // k values staged per LDS chunk

// a float known to sit in global memory (a pointer that went through an asm barrier would otherwise be loaded with
// address-space-generic instructions, whose completion the compiler cannot order against other loads)
typedef float __attribute__((address_space(1))) GlobalFloat;

__device__ inline float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// 16 consecutive k values of row `row` starting at k0 + 16*(lane/32); zero beyond n / K
template <bool BF16>
__device__ inline void load_a16(const void *A, int64_t row, int64_t n, int lda, int k0, int K, bool vec_ok, float scale,
                                float (&a)[16])
{
    const int kk = (threadIdx.x & 63) >> 5;
    const int kbase = k0 + 16 * kk;
    if (row >= n) {
#pragma unroll
        for (int s = 0; s < 16; ++s) a[s] = 0.0f;
        return;
    }
    if (BF16) {
        const uint16_t *p = static_cast<const uint16_t *>(A) + row * lda + kbase;
        if (vec_ok && kbase + 16 <= K) {
            const uint4 v0 = *reinterpret_cast<const uint4 *>(p);
            const uint4 v1 = *reinterpret_cast<const uint4 *>(p + 8);
            const uint32_t w[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                a[2 * i] = __uint_as_float(w[i] << 16) * scale;
                a[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u) * scale;
            }
        } else {
#pragma unroll
            for (int s = 0; s < 16; ++s) a[s] = kbase + s < K ? bf16_bits_to_f32(p[s]) * scale : 0.0f;
        }
    } else {
        const float *p = static_cast<const float *>(A) + row * lda + kbase;
        if (vec_ok && kbase + 16 <= K) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float4 v = *reinterpret_cast<const float4 *>(p + 4 * i);
                a[4 * i] = v.x * scale;
                a[4 * i + 1] = v.y * scale;
                a[4 * i + 2] = v.z * scale;
                a[4 * i + 3] = v.w * scale;
            }
        } else {
#pragma unroll
            for (int s = 0; s < 16; ++s) a[s] = kbase + s < K ? p[s] * scale : 0.0f;
        }
    }
}

// Stages W[k0 .. k0+32) x [cols] into LDS as Bs[kk][c], zero padded.  `col_of(c)` maps a staged column to a
// column of W (or -1).  Non-transposed W is [K, ldw]; transposed W is [M, ldw] and B[k][j] = W[j][k].
template <class ColOf>
__device__ inline void stage_b(float *Bs, int ldb, int ncols, const float *W, int ldw, bool wT, int k0, int K, ColOf col_of)
{
    const int total = kBK * ncols;
    if (!wT) {
        for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {
            const int kk = idx / ncols, c = idx - kk * ncols;
            const int wc = col_of(c);
            const int k = k0 + kk;
            Bs[kk * ldb + c] = (wc >= 0 && k < K) ? W[int64_t(k) * ldw + wc] : 0.0f;
        }
    } else {
        for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {
            const int c = idx / kBK, kk = idx - c * kBK;
            const int wc = col_of(c);
            const int k = k0 + kk;
            Bs[kk * ldb + c] = (wc >= 0 && k < K) ? W[int64_t(wc) * ldw + k] : 0.0f;
        }
    }
}

// Whole-slab staging for the LDS-resident kernels: Bs[k][c] (row length NC) for k in [0, K), where the NC
// staged columns are runs of RUN consecutive columns of W and run r starts at W column run_col(r).  A thread
// owns one 16-byte column position and walks down the rows with a fixed pointer stride, so a load costs two
// or three instructions; kStageDepth loads are in flight per thread and nothing is conditional (a row index
// past the end is clamped, which repeats a load and its store).  Needs 16-byte aligned rows of W (ldw % 4 == 0, aligned base,
// run starts % 4 == 0) and TPB >= NC / 4 threads.
constexpr int kStageDepth = 4;

template <int NC, int RUN, int TPB, class RunCol>
__device__ inline void stage_slab(float *Bs, const float *W, int ldw, int K, RunCol run_col)
{
    constexpr int V = NC / 4, RV = RUN / 4;
    constexpr int RPS = TPB / V;  // slab rows covered per step by the first RPS * V threads
    static_assert(RPS >= 1, "block too small for the slab width");
    const int tid = threadIdx.x;
    const int k0 = tid / V, c4 = tid - k0 * V;
    if (k0 >= RPS || k0 >= K) return;
    const int run = c4 / RV, off = c4 - run * RV;
    const float *src = W + int64_t(k0) * ldw + run_col(run) + 4 * off;
    float *dst = Bs + 4 * tid;
    const int last = (K - k0 - 1) / RPS;  // this thread stages rows k0 + RPS * (0 .. last)
    const int sstep = RPS * ldw;
    // rows beyond `last` repeat row `last`: duplicate loads and stores of one value instead of branches
    for (int b = 0; b <= last; b += kStageDepth) {
        float4 v[kStageDepth];
#pragma unroll
        for (int u = 0; u < kStageDepth; ++u) v[u] = *reinterpret_cast<const float4 *>(src + int64_t(min(b + u, last)) * sstep);
#pragma unroll
        for (int u = 0; u < kStageDepth; ++u) *reinterpret_cast<float4 *>(dst + min(b + u, last) * (4 * RPS * V)) = v[u];
    }
}

// The same for a transposed operand: Bs[k][j] = W[col0 + j][k] for j in [0, NC), W row-major [M, ldw].
// Lanes run along j, so the LDS stores of a wave fall into consecutive banks.  Needs K % 4 == 0.
template <int NC, int TPB>
__device__ inline void stage_slab_transposed(float *Bs, const float *W, int ldw, int K, int col0)
{
    constexpr int QPS = TPB / NC;  // k quads covered per step by the first QPS * NC threads
    static_assert(QPS >= 1, "block too small for the slab width");
    const int tid = threadIdx.x;
    const int q0 = tid / NC, j = tid - q0 * NC;
    if (q0 >= QPS || 4 * q0 >= K) return;
    const float *src = W + int64_t(col0 + j) * ldw + 4 * q0;
    float *dst = Bs + 4 * q0 * NC + j;
    const int last = (K / 4 - q0 - 1) / QPS;
    for (int b = 0; b <= last; b += kStageDepth) {
        float4 v[kStageDepth];
#pragma unroll
        for (int u = 0; u < kStageDepth; ++u) v[u] = *reinterpret_cast<const float4 *>(src + min(b + u, last) * (4 * QPS));
#pragma unroll
        for (int u = 0; u < kStageDepth; ++u) {
            float *d = dst + min(b + u, last) * (4 * QPS * NC);
            d[0] = v[u].x;
            d[NC] = v[u].y;
            d[2 * NC] = v[u].z;
            d[3 * NC] = v[u].w;
        }
    }
}

struct GemmArgs {
    const void *A;
    int64_t n;
    int K, M, lda;
    const float *row_scale;  // [n] or null
    const float *W;
    int ldw, wT;
    const float *bias;   // [M] or null
    int relu;
    const float *mask;   // [n, M] or null: output is zeroed where mask <= 0
    const float *add;    // [n, M] or null: added to the output
    float *out;          // [n, M]
};

// 4 waves as WM x WN; each wave owns 32 rows x (32*NT) columns.
template <int NT, int WM, int WN, bool BF16>
__global__ void __launch_bounds__(256) gemm_rows_kernel(GemmArgs g)
{
    constexpr int BN = 32 * NT * WN;
    constexpr int LDB = BN + 1;
    __shared__ float Bs[kBK * LDB];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int wm = w / WN, wn = w % WN;
    const int i = lane & 31, kk = lane >> 5;
    const int col0 = blockIdx.y * BN;
    const int64_t row = (int64_t(blockIdx.x) * WM + wm) * 32 + i;
    const bool vec_ok = (g.lda % (BF16 ? 8 : 4)) == 0;
    const float scale = (g.row_scale && row < g.n) ? g.row_scale[row] : 1.0f;
    acc16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
    for (int k0 = 0; k0 < g.K; k0 += kBK) {
        float a[16];
        load_a16<BF16>(g.A, row, g.n, g.lda, k0, g.K, vec_ok, scale, a);
        __syncthreads();
        stage_b(Bs, LDB, BN, g.W, g.ldw, g.wT != 0, k0, g.K, [&](int c) { return col0 + c < g.M ? col0 + c : -1; });
        __syncthreads();
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            const float *brow = Bs + (16 * kk + s) * LDB + wn * 32 * NT + i;
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], brow[32 * t], acc[t], 0, 0, 0);
        }
    }
    const int64_t rbase = (int64_t(blockIdx.x) * WM + wm) * 32;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int c = col0 + wn * 32 * NT + 32 * t + i;
        if (c >= g.M) continue;
        const float b = g.bias ? g.bias[c] : 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t rr = rbase + 8 * (r / 4) + 4 * kk + (r % 4);
            if (rr >= g.n) continue;
            float v = acc[t][r] + b;
            if (g.relu) v = fmaxf(v, 0.0f);
            if (g.add) v += g.add[rr * g.M + c];
            if (g.mask && !(g.mask[rr * g.M + c] > 0.0f)) v = 0.0f;
            g.out[rr * g.M + c] = v;
        }
    }
}

// 16 consecutive k values of row `row` (a valid row) starting at k0 + 16*(lane/32), as four 16-byte loads.
template <bool BF16>
__device__ inline void load_a16_fast(const void *A, int64_t row, int lda, int k0, float (&a)[16])
{
    const int kbase = k0 + 16 * ((threadIdx.x & 63) >> 5);
    if (BF16) {
        const uint16_t *p = static_cast<const uint16_t *>(A) + row * lda + kbase;
        const uint4 v0 = *reinterpret_cast<const uint4 *>(p);
        const uint4 v1 = *reinterpret_cast<const uint4 *>(p + 8);
        const uint32_t w[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a[2 * i] = __uint_as_float(w[i] << 16);
            a[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    } else {
        const float *p = static_cast<const float *>(A) + row * lda + kbase;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float4 v = *reinterpret_cast<const float4 *>(p + 4 * i);
            a[4 * i] = v.x;
            a[4 * i + 1] = v.y;
            a[4 * i + 2] = v.z;
            a[4 * i + 3] = v.w;
        }
    }
}

// The same from a ready pointer to the lane's first value.
template <bool BF16>
__device__ inline void load_a16_ptr(const char *p, float (&a)[16])
{
    if (BF16) {
        const uint4 v0 = *reinterpret_cast<const uint4 *>(p);
        const uint4 v1 = *reinterpret_cast<const uint4 *>(p + 16);
        const uint32_t w[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a[2 * i] = __uint_as_float(w[i] << 16);
            a[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float4 v = *reinterpret_cast<const float4 *>(p + 16 * i);
            a[4 * i] = v.x;
            a[4 * i + 1] = v.y;
            a[4 * i + 2] = v.z;
            a[4 * i + 3] = v.w;
        }
    }
}

// 16 k-steps against B fragments in LDS.  bp points at this lane's column of the first of its 16 B rows;
// tile t of NT sits at column offset tile_stride * t and accumulates into acc[t], except that the last tile
// accumulates into acc[LAST] (the recurrent step keeps one gate's two halves apart).  Fragments are read in
// groups of G steps ahead of their matrix instructions: the scheduling barriers keep the compiler from
// sinking each read next to its use, which would expose one LDS round trip per step.
template <int NT, int LAST, int G, int NACC, class Prefetch>
__device__ inline void mfma_chunk_map(const float (&a)[16], const float *bp, int ld, int tile_stride, acc16 (&acc)[NACC],
                                      Prefetch prefetch)
{
#pragma unroll
    for (int q = 0; q < 16 / G; ++q) {
        float b[G][NT];
#pragma unroll
        for (int s = 0; s < G; ++s)
#pragma unroll
            for (int t = 0; t < NT; ++t) b[s][t] = bp[(G * q + s) * ld + t * tile_stride];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < G; ++s)
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                constexpr int dummy = 0;
                (void)dummy;
                acc16 &dst = acc[t == NT - 1 ? LAST : t];
                dst = __builtin_amdgcn_mfma_f32_32x32x2f32(a[G * q + s], b[s][t], dst, 0, 0, 0);
            }
        if (q == 0) prefetch();
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int NT, class Prefetch>
__device__ inline void mfma_chunk(const float (&a)[16], const float *bp, int ld, int tile_stride, acc16 (&acc)[NT],
                                  Prefetch prefetch)
{
    mfma_chunk_map<NT, NT - 1, 8>(a, bp, ld, tile_stride, acc, prefetch);
}

struct NoPrefetch {
    __device__ void operator()() const {}
};

// ---- fp32 products on the bf16 matrix cores ---------------------------------------------------------------------
// An fp32 value is the sum of three bfloat16 terms, v = hi + mid + lo with |v - (hi + mid + lo)| <= 2^-24 |v|
// (each term is the round-to-nearest bfloat16 of what the terms before it leave over; the remainders are exact in
// fp32).  A product of two such sums, kept to the terms of relative size 2^-16 and above -- hi*hi, hi*mid, mid*hi,
// hi*lo, mid*mid, lo*hi -- is exact to about 2^-23 of |a*b|, and every one of the six is a bf16 x bf16 product that
// the matrix core forms exactly and adds in fp32.  Six bf16 instructions of depth 16 do the work of eight fp32
// instructions of depth 2 in 3/8 of the cycles.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ inline uint32_t pack_bf16(float a, float b)  // a in the low half; one v_cvt_pk_bf16_f32
{
    bf16x2 p;
    p[0] = static_cast<__bf16>(a);
    p[1] = static_cast<__bf16>(b);
    return __builtin_bit_cast(uint32_t, p);
}

// Splits eight consecutive values into their three bfloat16 planes (pairs packed low half first).
__device__ inline void split8(const float *v, u32x4 &hi, u32x4 &mid, u32x4 &lo)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float a0 = v[2 * j], a1 = v[2 * j + 1];
        uint32_t h = pack_bf16(a0, a1);
        asm volatile("" : "+v"(h));  // both halves come out of this one conversion (left alone, the low half gets a second one)
        const float r0 = a0 - __uint_as_float(h << 16), r1 = a1 - __uint_as_float(h & 0xFFFF0000u);
        uint32_t m = pack_bf16(r0, r1);
        asm volatile("" : "+v"(m));
        const float q0 = r0 - __uint_as_float(m << 16), q1 = r1 - __uint_as_float(m & 0xFFFF0000u);
        hi[j] = h;
        mid[j] = m;
        lo[j] = pack_bf16(q0, q1);
    }
}

__device__ inline acc16 mfma_bf16(u32x4 a, u32x4 b, acc16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Stages columns [col0, col0 + NC) of W (or of W^T) for the split product: for every group of eight k values and
// every column one 16-byte record per plane, planes[p][k / 8][column].  Columns at or beyond M are zero.
template <int NC, int TPB>
__device__ inline void stage_split(u32x4 *Bq, const float *W, int ldw, int K, bool wT, int col0, int M)
{
    const int groups = K / 8, plane = groups * NC;
    const bool vec = wT && ldw % 4 == 0 && (reinterpret_cast<uintptr_t>(W) & 15) == 0;
    for (int item = threadIdx.x; item < plane; item += TPB) {
        const int g8 = item / NC, c = col0 + item % NC;
        float v[8];
        if (c >= M) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = 0.0f;
        } else if (!wT) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = W[int64_t(8 * g8 + e) * ldw + c];
        } else if (vec) {
            const float4 x = *reinterpret_cast<const float4 *>(W + int64_t(c) * ldw + 8 * g8);
            const float4 y = *reinterpret_cast<const float4 *>(W + int64_t(c) * ldw + 8 * g8 + 4);
            v[0] = x.x, v[1] = x.y, v[2] = x.z, v[3] = x.w, v[4] = y.x, v[5] = y.y, v[6] = y.z, v[7] = y.w;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = W[int64_t(c) * ldw + 8 * g8 + e];
        }
        u32x4 h, m, l;
        split8(v, h, m, l);
        Bq[item] = h;
        Bq[plane + item] = m;
        Bq[2 * plane + item] = l;
    }
}

// The same for K rows of a row-major W whose slab columns are picked by col_of(c) (a source column, or -1 for a
// column of zeros); the rows become groups group0 .. group0 + K/8 - 1 of a slab of `plane` records per plane.
template <int NC, int TPB, class ColOf>
__device__ inline void stage_split_cols(u32x4 *Bq, int plane, int group0, const float *W, int ldw, int K, ColOf col_of)
{
    for (int item = threadIdx.x; item < K / 8 * NC; item += TPB) {
        const int g8 = item / NC, c = col_of(item % NC);
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = c >= 0 ? W[int64_t(8 * g8 + e) * ldw + c] : 0.0f;
        u32x4 h, m, l;
        split8(v, h, m, l);
        u32x4 *dst = Bq + group0 * NC + item;
        dst[0] = h;
        dst[plane] = m;
        dst[2 * plane] = l;
    }
}

// One 32-deep chunk of the split product: the lane's 16 values of A are two groups of eight k values, each split into
// three planes and multiplied with the staged planes of W, smallest terms first.  bq points at this lane's record of
// the chunk's first group of plane 0; consecutive groups are `ld` records apart, planes `plane` records, the wave's
// NT column tiles `tile_stride` records; tile t accumulates into acc[t].
template <int NT, int NACC>
__device__ inline void mfma_chunk_split(const float (&a)[16], const u32x4 *bq, int ld, int plane, int tile_stride, acc16 (&acc)[NACC])
{
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        u32x4 b0[NT], b1[NT], b2[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            b0[t] = bq[m * ld + tile_stride * t];
            b1[t] = bq[plane + m * ld + tile_stride * t];
            b2[t] = bq[2 * plane + m * ld + tile_stride * t];
        }
        u32x4 ah, am, al;
        split8(a + 8 * m, ah, am, al);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = mfma_bf16(al, b0[t], acc[t]);
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = mfma_bf16(am, b1[t], acc[t]);
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = mfma_bf16(ah, b2[t], acc[t]);
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = mfma_bf16(am, b0[t], acc[t]);
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = mfma_bf16(ah, b1[t], acc[t]);
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = mfma_bf16(ah, b0[t], acc[t]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Same product with the whole weight slab [K, 32*NT*WN] resident in LDS: it is staged once per block, after
// which every wave streams its own 32-row tiles without any barrier.  A block is as many waves as the
// register budget of the variant allows (one block per compute unit), so the slab is fetched once per compute
// unit and even a slab that fills the LDS leaves the unit fully occupied.  The k chunks of all of a wave's
// tiles form one stream; a ring of three register buffers keeps the loads two chunks (8 KB per wave) ahead of
// the matrix cores, across tile boundaries and epilogues.  Needs K % 32 == 0 and 16-byte aligned rows; the
// row scale is applied to the rows of A as they are consumed.  SPLIT: the slab holds the three bfloat16 planes of
// the weights (6 bytes per value instead of 4) and the product runs on the bf16 matrix cores, see above.
template <int NT, int WN, int WAVES, bool BF16, bool SPLIT>
__global__ void __launch_bounds__(64 * WAVES) gemm_rows_resident_kernel(GemmArgs g)
{
    // WAVES waves = (WAVES / WN) row tiles x WN column groups of 32*NT columns; the slab holds all 32*NT*WN columns
    extern __shared__ float Bs[];
    constexpr int BN = 32 * NT * WN;
    constexpr int WR = WAVES / WN;
    static_assert(WAVES % WN == 0, "column groups must divide the block");
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int wn = w % WN, wr = w / WN;
    const int i = lane & 31, kk = lane >> 5;
    const int col0 = blockIdx.y * BN;
    // tile indices fit 32 bits (n < 2^31 rows); all cursor arithmetic is wave-uniform
    const int ntiles = int((g.n + 31) / 32);
    const int first = __builtin_amdgcn_readfirstlane(int(blockIdx.x) * WR + wr), stride = int(gridDim.x) * WR;
    const int kch = g.K / kBK;
    const float *bp0 = Bs + (16 * kk) * BN + wn * 32 * NT + i;
    u32x4 *Bq = reinterpret_cast<u32x4 *>(Bs);
    const int plane = g.K / 8 * BN;                         // records per plane of the split slab
    const u32x4 *bq0 = Bq + (2 * kk) * BN + wn * 32 * NT + i;  // this lane's record of group 2*kk (chunk 0), plane 0
    const int wcol0 = col0 + wn * 32 * NT;
    constexpr int ES = BF16 ? 2 : 4;
    auto row_ptr = [&](int t) __attribute__((always_inline)) {  // this lane's 16 k values of chunk 0 in tile t
        return static_cast<const char *>(g.A) + (min(int64_t(t) * 32 + i, g.n - 1) * g.lda + 16 * kk) * ES;
    };

    // The row scale travels with the chunk: every lane loads the scale of its row next to its 16 k values and
    // multiplies them before the matrix instructions (a load in the epilogue would make the wave wait for
    // everything in flight, once per tile).  Without a row scale the same load reads a valid dummy address and
    // the factor is 1: the load stays unconditional, which keeps the waits on the ring exact.
    const bool has_rs = g.row_scale != nullptr;
    auto scale_ptr = [&](int t) __attribute__((always_inline)) {
        return has_rs ? g.row_scale + min(int64_t(t) * 32 + i, g.n - 1) : static_cast<const float *>(g.A);
    };

    // load cursor: chunk lk of tile ltile
    int ltile = first, lk = 0;
    const char *lptr = row_ptr(ltile < ntiles ? ltile : 0);
    const float *lsp = scale_ptr(ltile < ntiles ? ltile : 0);
    auto issue = [&](float(&buf)[16], float &sc) __attribute__((always_inline)) {
        if (ltile < ntiles) {
            load_a16_ptr<BF16>(lptr, buf);
            asm volatile("" : "+v"(lsp));  // one scale load per chunk, never merged into a per-tile (conditional) one
            sc = *(const GlobalFloat *)lsp;
            lptr += kBK * ES;
            if (++lk == kch) {
                lk = 0;
                ltile += stride;
                if (ltile < ntiles) {
                    lptr = row_ptr(ltile);
                    lsp = scale_ptr(ltile);
                }
            }
        }
    };
    auto issue_always = [&](float(&buf)[16], float &sc) __attribute__((always_inline)) {  // the caller knows that the chunk exists
        load_a16_ptr<BF16>(lptr, buf);
        asm volatile("" : "+v"(lsp));
        sc = *(const GlobalFloat *)lsp;
        lptr += kBK * ES;
        if (++lk == kch) {
            lk = 0;
            ltile += stride;
            lptr = row_ptr(ltile);
            lsp = scale_ptr(ltile);
        }
    };
    // the first two chunks of A are requested before the weight slab is staged: both fetches overlap
    float b0[16], b1[16], b2[16], s0 = 1.0f, s1 = 1.0f, s2 = 1.0f;
    issue(b0, s0);
    issue(b1, s1);
    const bool fast_stage = col0 + BN <= g.M && g.ldw % 4 == 0 && (reinterpret_cast<uintptr_t>(g.W) & 15) == 0;
    if (SPLIT) {
        stage_split<BN, 64 * WAVES>(Bq, g.W, g.ldw, g.K, g.wT != 0, col0, g.M);
    } else if (fast_stage && !g.wT) {
        stage_slab<BN, BN, 64 * WAVES>(Bs, g.W, g.ldw, g.K, [&](int) { return col0; });
    } else if (fast_stage) {
        stage_slab_transposed<BN, 64 * WAVES>(Bs, g.W, g.ldw, g.K, col0);
    } else {
        for (int k0 = 0; k0 < g.K; k0 += kBK)
            stage_b(Bs + k0 * BN, BN, BN, g.W, g.ldw, g.wT != 0, k0, g.K, [&](int c) { return col0 + c < g.M ? col0 + c : -1; });
    }
    __syncthreads();
    // everything requested so far has landed by now; saying so keeps the waits inside the loops exact
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    // compute cursor
    int tile = first, kc = 0;
    float bias[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) bias[t] = (g.bias && wcol0 + 32 * t + i < g.M) ? g.bias[wcol0 + 32 * t + i] : 0.0f;
    acc16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;

    auto epilogue = [&]() __attribute__((always_inline)) {  // rows rbase + 8*q + e (q, e in 0..3) of the finished tile, four rows at a time
        const int64_t rbase = int64_t(tile) * 32 + 4 * kk;
        const bool full = int64_t(tile) * 32 + 32 <= g.n;
        if (full) {
            // a whole tile: an element's address is a wave-uniform part (tile and row inside it: scalar arithmetic) plus
            // a lane part that never changes (row half and column), so no vector instruction goes into addressing
            const uint32_t row_bytes = uint32_t(g.M) * 4u;
            const int64_t tile_off = int64_t(tile) * 32 * row_bytes;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int c = wcol0 + 32 * t + i;
                if (c < g.M) {
                    const uint32_t lane_off = uint32_t(4 * kk) * row_bytes + uint32_t(c) * 4u;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float v[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            v[e] = acc[t][4 * q + e] + bias[t];
                            if (g.relu) v[e] = fmaxf(v[e], 0.0f);
                        }
                        if (g.add) {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                v[e] += *reinterpret_cast<const float *>(reinterpret_cast<const char *>(g.add) + tile_off +
                                                                         uint32_t(8 * q + e) * row_bytes + lane_off);
                        }
                        if (g.mask) {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (!(*reinterpret_cast<const float *>(reinterpret_cast<const char *>(g.mask) + tile_off +
                                                                       uint32_t(8 * q + e) * row_bytes + lane_off) > 0.0f))
                                    v[e] = 0.0f;
                        }
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            *reinterpret_cast<float *>(reinterpret_cast<char *>(g.out) + tile_off + uint32_t(8 * q + e) * row_bytes +
                                                       lane_off) = v[e];
                    }
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
            }
            return;
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int c = wcol0 + 32 * t + i;
            if (c < g.M) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    int64_t o[4];
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int64_t rr = min(rbase + 8 * q + e, g.n - 1);
                        o[e] = rr * g.M + c;
                        v[e] = acc[t][4 * q + e] + bias[t];
                        if (g.relu) v[e] = fmaxf(v[e], 0.0f);
                    }
                    if (g.add) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += g.add[o[e]];
                    }
                    if (g.mask) {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (!(g.mask[o[e]] > 0.0f)) v[e] = 0.0f;
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (full || rbase + 8 * q + e < g.n) g.out[o[e]] = v[e];
                }
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
        }
    };
    auto multiply = [&](float(&cur)[16], float sc) __attribute__((always_inline)) {
        const float f = has_rs ? sc : 1.0f;
#pragma unroll
        for (int e = 0; e < 16; ++e) cur[e] *= f;
        if (SPLIT)
            mfma_chunk_split<NT, NT>(cur, bq0 + kc * 4 * BN, BN, plane, 32, acc);
        else
            mfma_chunk<NT>(cur, bp0 + kc * kBK * BN, BN, 32, acc, NoPrefetch());
        if (++kc == kch) {
            epilogue();
            kc = 0;
            tile += stride;
        }
    };
    // Steady state: while the chunk two ahead of the one being multiplied exists, its load is unconditional,
    // so the wait in front of a chunk's matrix instructions covers exactly the loads older than the last two.
    // (A load that may or may not have been issued forces a wait for everything.)
    const int my_tiles = first < ntiles ? (ntiles - first + stride - 1) / stride : 0;
    const int steady = max(my_tiles * kch - 2, 0) / 3;
    for (int j = 0; j < steady; ++j) {
        issue_always(b2, s2);
        __builtin_amdgcn_sched_barrier(0);  // the new loads go out before this chunk's matrix instructions
        multiply(b0, s0);
        issue_always(b0, s0);
        __builtin_amdgcn_sched_barrier(0);
        multiply(b1, s1);
        issue_always(b1, s1);
        __builtin_amdgcn_sched_barrier(0);
        multiply(b2, s2);
    }
    // the last chunks: loads only while chunks remain
    auto step = [&](float(&cur)[16], float &csc, float(&nxt)[16], float &nsc) __attribute__((always_inline)) {
        const float sc = csc;
        issue(nxt, nsc);
        __builtin_amdgcn_sched_barrier(0);
        multiply(cur, sc);
    };
    while (tile < ntiles) {
        step(b0, s0, b2, s2);
        if (tile < ntiles) step(b1, s1, b0, s0);
        if (tile < ntiles) step(b2, s2, b1, s1);
    }
}

constexpr int kNumCU = 256;
constexpr size_t kLdsBytes = 160 * 1024;

// blocks of this kernel that fit on one compute unit at once (registers and LDS); the persistent grids are
// sized with it so that every block is resident from the start
int resident_blocks(const void *kernel, int threads, size_t lds)
{
    int blocks = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, kernel, threads, lds) != hipSuccess) return 0;
    return blocks;
}

template <int NT, int WN, int WAVES, bool SPLIT>
bool gemm_rows_resident_launch(const GemmArgs &g, int bf16, hipStream_t s)
{
    if (g.K % kBK != 0 || g.lda % 8 != 0) return false;
    constexpr int BN = 32 * NT * WN;
    const size_t lds = size_t(g.K) * BN * (SPLIT ? 6 : sizeof(float));
    if (lds > kLdsBytes - 1024) return false;
    auto k = bf16 ? gemm_rows_resident_kernel<NT, WN, WAVES, true, SPLIT> : gemm_rows_resident_kernel<NT, WN, WAVES, false, SPLIT>;
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, int(lds)) != hipSuccess)
        return false;
    const int per_cu = resident_blocks(reinterpret_cast<const void *>(k), 64 * WAVES, lds);
    if (per_cu <= 0) return false;
    const int64_t ntiles = (g.n + 31) / 32;
    constexpr int wr = WAVES / WN;
    const unsigned gy = unsigned((g.M + BN - 1) / BN);
    dim3 grid(unsigned(std::min<int64_t>((ntiles + wr - 1) / wr, std::max<int64_t>(1, int64_t(kNumCU) * per_cu / gy))), gy);
    k<<<grid, 64 * WAVES, lds, s>>>(g);
    return true;
}

// REINC_DENSE=fp32 keeps every dense product on the fp32 matrix instructions (the split-bf16 kernels are the default)
bool dense_split_enabled()
{
    static const bool on = [] {
        const char *v = getenv("REINC_DENSE");
        return !(v && strcmp(v, "fp32") == 0);
    }();
    return on;
}

// Variant choice (measured on 1e5 .. 2.5e6 rows, K and M in 64 .. 512): the widest accumulator tile whose slab
// fits wins for outputs of more than 64 columns; when the slab of 128 columns does not fit, 64-column slabs
// with the column groups on blockIdx.y follow (A is then re-read out of L2).  The split-bf16 variants come first;
// shapes whose three-plane slab does not fit (K * columns * 6 bytes) stay on the fp32 instructions.
bool gemm_rows_resident_dispatch(const GemmArgs &g, int bf16, hipStream_t s)
{
    if (dense_split_enabled()) {
        if (g.M > 64 && gemm_rows_resident_launch<4, 1, 8, true>(g, bf16, s)) return true;
        if (g.M > 64 && gemm_rows_resident_launch<2, 1, 12, true>(g, bf16, s)) return true;
        if (g.M > 32 && g.M <= 64 && gemm_rows_resident_launch<2, 1, 12, true>(g, bf16, s)) return true;  // 16 waves would spill
        if (g.M <= 32 && gemm_rows_resident_launch<1, 1, 16, true>(g, bf16, s)) return true;
        // (deep products such as K = 512 -> 128 would fit a 32-column split slab only; four column groups re-splitting
        // the same rows were measured no faster than the fp32 instructions with a 64-column slab)
    }
    if (g.M > 64 && gemm_rows_resident_launch<4, 1, 8, false>(g, bf16, s)) return true;
    if (g.M > 64 && gemm_rows_resident_launch<2, 1, 12, false>(g, bf16, s)) return true;
    if (g.M > 32 && g.M <= 64 && gemm_rows_resident_launch<2, 1, 16, false>(g, bf16, s)) return true;
    return gemm_rows_resident_launch<1, 1, 16, false>(g, bf16, s);
}

template <int NT, int WM, int WN>
void gemm_rows_launch(const GemmArgs &g, int bf16, hipStream_t s)
{
    constexpr int BN = 32 * NT * WN;
    dim3 grid(unsigned((g.n + 32 * WM - 1) / (32 * WM)), unsigned((g.M + BN - 1) / BN));
    if (bf16)
        gemm_rows_kernel<NT, WM, WN, true><<<grid, 256, 0, s>>>(g);
    else
        gemm_rows_kernel<NT, WM, WN, false><<<grid, 256, 0, s>>>(g);
}

// ---- fused recurrent step ----------------------------------------------------------------------------------
struct RnnArgs {
    const float *x;
    int64_t n;
    int d_in, H;
    const float *h_prev, *c_prev;  // may be null (zero state)
    const float *x_scale;          // [n] or null: every row of x is multiplied by its scale first
    const float *h_carry;          // GRU: the state in the carry term z .* h (normally h_prev itself; null = zero)
    const float *W_i, *W_h, *b_i, *b_h;
    float *h_out, *c_out, *saved;
};

// Gate activations on the hardware exp2 / reciprocal instructions (about 1 ulp each): absolute error below
// 3e-7, far inside the 1e-4 tolerance on the step's outputs, at a fifth of the instructions of expf/tanhf.
__device__ inline float sigmoidf_(float v) { return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504f * v)); }
__device__ inline float tanhf_(float v) { return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(2.88539008f * v)); }

// 4 waves as WM x WN; each wave owns 32 rows x 32 hidden units and four 32x32 accumulators:
//   LSTM: gates i, f, g, o (x and h parts summed);   GRU: r, z (summed), x-part of n, h-part of n.
template <bool LSTM, int WM, int WN>
__global__ void __launch_bounds__(256) rnn_fused_kernel(RnnArgs g)
{
    constexpr int KG = LSTM ? 4 : 3;
    constexpr int BH = 32 * WN;  // hidden units per block
    constexpr int NC = KG * BH;
    constexpr int LDB = NC;  // reads walk consecutive columns, so no padding is needed
    __shared__ float Bs[kBK * LDB];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int wm = w / WN, wn = w % WN;
    const int i = lane & 31, kk = lane >> 5;
    const int h0 = blockIdx.y * BH;
    const int64_t row = (int64_t(blockIdx.x) * WM + wm) * 32 + i;
    const int H = g.H, ldw = KG * H;
    acc16 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
    auto col_of = [&](int c) {
        const int gate = c / BH, j = c - gate * BH;
        return h0 + j < H ? gate * H + h0 + j : -1;
    };
    for (int part = 0; part < 2; ++part) {
        const float *A = part == 0 ? g.x : g.h_prev;
        if (!A) continue;  // zero recurrent state: the h part contributes nothing
        const int K = part == 0 ? g.d_in : H;
        const float *W = part == 0 ? g.W_i : g.W_h;
        const bool vec_ok = (K % 4) == 0;
        for (int k0 = 0; k0 < K; k0 += kBK) {
            float a[16];
            const float sc = (part == 0 && g.x_scale && row < g.n) ? g.x_scale[row] : 1.0f;
            load_a16<false>(A, row, g.n, K, k0, K, vec_ok, sc, a);
            __syncthreads();
            stage_b(Bs, LDB, NC, W, ldw, false, k0, K, col_of);
            __syncthreads();
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                const float *brow = Bs + (16 * kk + s) * LDB + wn * 32 + i;
                if (LSTM) {
#pragma unroll
                    for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], brow[t * BH], acc[t], 0, 0, 0);
                } else {
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], brow[0], acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], brow[BH], acc[1], 0, 0, 0);
                    if (part == 0)
                        acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], brow[2 * BH], acc[2], 0, 0, 0);
                    else
                        acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], brow[2 * BH], acc[3], 0, 0, 0);
                }
            }
        }
    }
    const int j = h0 + wn * 32 + i;
    if (j >= H) return;
    const int64_t rbase = (int64_t(blockIdx.x) * WM + wm) * 32;
    float bi[KG], bh[KG];
#pragma unroll
    for (int t = 0; t < KG; ++t) {
        bi[t] = g.b_i ? g.b_i[t * H + j] : 0.0f;
        bh[t] = g.b_h ? g.b_h[t * H + j] : 0.0f;
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int64_t rr = rbase + 8 * (r / 4) + 4 * kk + (r % 4);
        if (rr >= g.n) continue;
        const int64_t o = rr * H + j;
        if (LSTM) {
            const float gi = sigmoidf_(acc[0][r] + bi[0] + bh[0]);
            const float gf = sigmoidf_(acc[1][r] + bi[1] + bh[1]);
            const float gg = tanhf_(acc[2][r] + bi[2] + bh[2]);
            const float go = sigmoidf_(acc[3][r] + bi[3] + bh[3]);
            const float cp = g.c_prev ? g.c_prev[o] : 0.0f;
            const float cn = gf * cp + gi * gg;
            g.c_out[o] = cn;
            g.h_out[o] = go * tanhf_(cn);
            if (g.saved) {
                float *sv = g.saved + rr * 4 * H + j;
                sv[0] = gi;
                sv[H] = gf;
                sv[2 * H] = gg;
                sv[3 * H] = go;
            }
        } else {
            const float gr = sigmoidf_(acc[0][r] + bi[0] + bh[0]);
            const float gz = sigmoidf_(acc[1][r] + bi[1] + bh[1]);
            const float ghn = acc[3][r] + bh[2];
            const float gn = tanhf_(acc[2][r] + bi[2] + gr * ghn);
            const float hp = g.h_carry ? g.h_carry[o] : 0.0f;
            g.h_out[o] = (1.0f - gz) * gn + gz * hp;
            if (g.saved) {
                float *sv = g.saved + rr * 4 * H + j;
                sv[0] = gr;
                sv[H] = gz;
                sv[2 * H] = gn;
                sv[3 * H] = ghn;
            }
        }
    }
}

// Same step with both weight matrices (the block's hidden-unit columns of every gate) resident in LDS:
// staged once per block (one block per compute unit), then every wave streams 32-row tiles for its 32 hidden
// units without barriers.  Rows [0, d_in) of the slab hold W_i, rows [d_in, d_in + H) hold W_h, so the k
// chunks of x and of h_prev form one stream per tile, and the chunks of all of a wave's tiles one stream
// overall; a ring of register buffers (three, four in the split variants) keeps the loads ahead of the matrix cores.  Needs
// d_in % 32 == 0, H % 32 == 0 and 16-byte aligned rows.  SPLIT: the slab holds the three bfloat16 planes of the
// weights and the products run on the bf16 matrix cores (see the note on fp32 products above).
//
// PACK (LSTM, split only): a wave takes 16 hidden units instead of 32 and packs two gates into each 32-column tile
// ([i | f] and [g | o]), so the slab is half as wide and fits the LDS where the unpacked one does not
// (d_in + H = 256: 98 KB instead of 196 KB).  The four gates of a hidden unit then sit in two lanes 16 apart; in the
// epilogue the two lanes swap half of their rows, after which each finishes its unit for 8 of the tile's 16 rows.
template <bool LSTM, int WN, int WAVES, bool SPLIT, bool PACK = false>
__global__ void __launch_bounds__(64 * WAVES) rnn_fused_resident_kernel(RnnArgs g)
{
    extern __shared__ float Bs[];
    static_assert(!PACK || (LSTM && SPLIT), "gate packing is for the split LSTM cell");
    constexpr int KG = LSTM ? 4 : 3;
    constexpr int WM = WAVES / WN;
    constexpr int UW = PACK ? 16 : 32;  // hidden units per wave
    constexpr int BH = UW * WN;
    constexpr int NC = KG * BH;
    constexpr int G = 4;  // B fragments are read four steps (12 or 16 registers) ahead
    static_assert(WAVES % WN == 0, "column groups must divide the block");
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int wm = w / WN, wn = w % WN;
    const int i = lane & 31, kk = lane >> 5;
    const int h0 = blockIdx.y * BH;
    const int H = g.H, ldw = KG * H;
    const int ntiles = int((g.n + 31) / 32);
    const int first = __builtin_amdgcn_readfirstlane(int(blockIdx.x) * WM + wm), stride = int(gridDim.x) * WM;
    // PACK: the previous state c_prev that the epilogue needs comes in as one more chunk of the tile's stream and is
    // moved into accumulator layout by the matrix cores (a product with an identity matrix, exact term by term).
    // Loads issued by the epilogue itself are waited for on the spot, once per tile, together with every load of the
    // ring.  (The unpacked variants have no registers left for a fifth accumulator: with it they spilled and took
    // half as long again.)
    const float *pstate = LSTM ? g.c_prev : g.h_carry;
    const int ks = (PACK && pstate) ? 1 : 0;
    const int kx = g.d_in / kBK, kh = g.h_prev ? H / kBK : 0, kch = kx + kh + ks;
    auto s_ptr = [&](int t) __attribute__((always_inline)) {  // the wave's 16 units, in both halves of the wave
        return reinterpret_cast<const char *>(pstate) + (min(int64_t(t) * 32 + i, g.n - 1) * H + h0 + wn * 16) * 4;
    };
    auto x_ptr = [&](int t) __attribute__((always_inline)) {
        return reinterpret_cast<const char *>(g.x) + (min(int64_t(t) * 32 + i, g.n - 1) * g.d_in + 16 * kk) * 4;
    };
    auto h_ptr = [&](int t) __attribute__((always_inline)) {
        return reinterpret_cast<const char *>(g.h_prev) + (min(int64_t(t) * 32 + i, g.n - 1) * H + 16 * kk) * 4;
    };
    // the row scale of x travels with its chunks (see gemm_rows_resident_kernel); chunks of h_prev carry a 1
    const bool has_xs = g.x_scale != nullptr;
    auto xs_ptr = [&](int t) __attribute__((always_inline)) {
        return has_xs ? g.x_scale + min(int64_t(t) * 32 + i, g.n - 1) : g.x;
    };
    // load cursor: chunk lk of tile ltile (chunks 0 .. kx-1 come from x, the rest from h_prev)
    int ltile = first, lk = 0;
    const char *lptr = x_ptr(ltile < ntiles ? ltile : 0);
    const float *lsp = xs_ptr(ltile < ntiles ? ltile : 0);
    auto advance = [&](bool more) __attribute__((always_inline)) {
        lptr += kBK * 4;
        ++lk;
        if (lk == kx && kh > 0) lptr = h_ptr(ltile);
        if (PACK && ks && lk == kx + kh) lptr = s_ptr(ltile);
        if (lk == kch) {
            lk = 0;
            ltile += stride;
            if (more) {
                lptr = x_ptr(ltile);
                lsp = xs_ptr(ltile);
            }
        }
    };
    auto issue = [&](float(&buf)[16], float &sc) __attribute__((always_inline)) {
        if (ltile < ntiles) {
            load_a16_ptr<false>(lptr, buf);
            asm volatile("" : "+v"(lsp));  // one scale load per chunk, never merged into a conditional one
            sc = *(const GlobalFloat *)lsp;
            advance(ltile + stride < ntiles || lk + 1 < kch);
        }
    };
    auto issue_always = [&](float(&buf)[16], float &sc) __attribute__((always_inline)) {  // the caller knows that the chunk exists
        load_a16_ptr<false>(lptr, buf);
        asm volatile("" : "+v"(lsp));
        sc = *(const GlobalFloat *)lsp;
        advance(true);
    };
    // A ring of RING register buffers keeps the loads RING - 1 chunks ahead of the matrix cores.  The split variants
    // have registers to spare (two waves per SIMD) and take four: on small graphs a wave has a handful of tiles
    // and its time is the chain of memory round trips, which a ring that holds a whole tile's chunks shortens.
    // The first chunks are requested before the slabs are staged: the fetches overlap.
    constexpr int RING = SPLIT ? 4 : 3;
    float buf[RING][16], bsc[RING];
#pragma unroll
    for (int r = 0; r < RING; ++r) bsc[r] = 1.0f;
#pragma unroll
    for (int r = 0; r + 1 < RING; ++r) issue(buf[r], bsc[r]);
    const bool fast_stage = h0 + BH <= H && H % 4 == 0 && (reinterpret_cast<uintptr_t>(g.W_i) & 15) == 0 &&
                            (reinterpret_cast<uintptr_t>(g.W_h) & 15) == 0;
    u32x4 *Bq = reinterpret_cast<u32x4 *>(Bs);
    const int plane = (g.d_in + H) / 8 * NC;  // records per plane of the split slab
    if (SPLIT) {
        auto col_of = [&](int c) {
            if (PACK) {  // a wave's 64 columns: its 16 units of gate i, then f, g, o
                const int wv = c / 64, r = c - wv * 64, gate = r / 16, unit = h0 + 16 * wv + (r & 15);
                return unit < H ? gate * H + unit : -1;
            }
            const int gate = c / BH, jj = c - gate * BH;
            return h0 + jj < H ? gate * H + h0 + jj : -1;
        };
        stage_split_cols<NC, 64 * WAVES>(Bq, plane, 0, g.W_i, ldw, g.d_in, col_of);
        stage_split_cols<NC, 64 * WAVES>(Bq, plane, g.d_in / 8, g.W_h, ldw, H, col_of);
    } else if (fast_stage) {
        stage_slab<NC, BH, 64 * WAVES>(Bs, g.W_i, ldw, g.d_in, [&](int gate) { return gate * H + h0; });
        stage_slab<NC, BH, 64 * WAVES>(Bs + int64_t(g.d_in) * NC, g.W_h, ldw, H, [&](int gate) { return gate * H + h0; });
    } else {
        auto col_of = [&](int c) {
            const int gate = c / BH, j = c - gate * BH;
            return h0 + j < H ? gate * H + h0 + j : -1;
        };
        for (int k0 = 0; k0 < g.d_in; k0 += kBK) stage_b(Bs + k0 * NC, NC, NC, g.W_i, ldw, false, k0, g.d_in, col_of);
        for (int k0 = 0; k0 < H; k0 += kBK) stage_b(Bs + (g.d_in + k0) * NC, NC, NC, g.W_h, ldw, false, k0, H, col_of);
    }
    __syncthreads();
    // everything requested so far has landed by now; saying so keeps the waits inside the loops exact
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    const int j = PACK ? h0 + wn * 16 + (i & 15) : h0 + wn * 32 + i;
    float bsum[KG], bhn = 0.0f;  // gate biases: b_i + b_h, except that GRU keeps b_hn apart (the reset gate scales it)
#pragma unroll
    for (int t = 0; t < KG; ++t) {
        const float bi = (g.b_i && j < H) ? g.b_i[t * H + j] : 0.0f;
        const float bh = (g.b_h && j < H) ? g.b_h[t * H + j] : 0.0f;
        if (!LSTM && t == 2) {
            bsum[t] = bi;
            bhn = bh;
        } else {
            bsum[t] = bi + bh;
        }
    }
    const float *bp0 = Bs + (16 * kk) * NC + wn * 32 + i;
    // compute cursor; accumulators: LSTM i, f, g, o (x and h parts summed); GRU r, z (summed), h part of n, x part of n;
    // PACK: [i | f], [g | o], the previous state
    int tile = first, kc = 0;
    acc16 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
    // identity fragment for the state chunk: the lane's eight k slots are the units 8 * kk + s of the wave, s = 0 .. 7,
    // and its column is unit i % 16, in both halves of the tile
    u32x4 ident;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int s1 = (i & 15) - 8 * kk;
        ident[e] = s1 == 2 * e ? 0x00003F80u : s1 == 2 * e + 1 ? 0x3F800000u : 0u;
    }

    auto epilogue = [&]() __attribute__((always_inline)) {  // rows rbase + 8*q + e of the finished tile, four at a time
        const int64_t rbase = int64_t(tile) * 32 + 4 * kk;
        const bool full = int64_t(tile) * 32 + 32 <= g.n;
        if (PACK) {
            // lanes 0..15 of a half hold gates i (acc[0]) and g (acc[1]) of their unit, lanes 16..31 gates f and o, for
            // the same 16 rows.  The low lane keeps rows 0..7 (registers 0..7) and receives f, o for them; the high
            // lane keeps rows 8..15 and receives i, g.
            // (The registers are made opaque first: a select between two elements of an accumulator would otherwise be
            // turned into one element at a selected index, which costs a chain of 15 selects per value.)
            const bool low = i < 16;
            float mine0[8], mine1[8], other0[8], other1[8], state[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                float a0 = acc[0][r], b0 = acc[0][8 + r], a1 = acc[1][r], b1 = acc[1][8 + r], a2 = acc[2][r], b2 = acc[2][8 + r];
                asm volatile("" : "+v"(a0), "+v"(b0), "+v"(a1), "+v"(b1), "+v"(a2), "+v"(b2));
                mine0[r] = low ? a0 : b0;
                mine1[r] = low ? a1 : b1;
                state[r] = low ? a2 : b2;
                other0[r] = __shfl_xor(low ? b0 : a0, 16);
                other1[r] = __shfl_xor(low ? b1 : a1, 16);
            }
            // the cell of row r (register index) from the exchanged gates; at(base, w) is this lane's element of its row
            // in a matrix of w * H columns
            auto packed_cell = [&](int r, float prev, auto at) __attribute__((always_inline)) {
                const float gi = sigmoidf_((low ? mine0[r] : other0[r]) + bsum[0]);
                const float gf = sigmoidf_((low ? other0[r] : mine0[r]) + bsum[1]);
                const float gg = tanhf_((low ? mine1[r] : other1[r]) + bsum[2]);
                const float go = sigmoidf_((low ? other1[r] : mine1[r]) + bsum[LSTM ? 3 : 0]);
                const float cn = gf * prev + gi * gg;
                *at(g.c_out, 1) = cn;
                *at(g.h_out, 1) = go * tanhf_(cn);
                if (g.saved) {
                    float *sv = at(g.saved, 4);
                    sv[0] = gi;
                    sv[H] = gf;
                    sv[2 * H] = gg;
                    sv[3 * H] = go;
                }
            };
            if (j < H && full) {
                // a whole tile: an element's address is a wave-uniform part (tile, row inside it) plus a lane part that
                // never changes (row half, lane half, unit), so addressing costs scalar arithmetic only
                const uint32_t hrow = uint32_t(H) * 4u;
                const int64_t tile_h = int64_t(tile) * 32 * hrow;
                const uint32_t lane_rows = uint32_t(4 * kk + (low ? 0 : 16));
                const uint32_t lane_h = lane_rows * hrow + uint32_t(j) * 4u, lane_s = lane_rows * 4u * hrow + uint32_t(j) * 4u;
#pragma unroll
                for (int q = 0; q < 2; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int64_t oh = tile_h + uint32_t(8 * q + e) * hrow;
                        packed_cell(4 * q + e, state[4 * q + e], [&](float *base, int w) __attribute__((always_inline)) {
                            return reinterpret_cast<float *>(reinterpret_cast<char *>(base) + w * oh + (w == 4 ? lane_s : lane_h));
                        });
                    }
            } else if (j < H) {
#pragma unroll
                for (int q = 0; q < 2; ++q) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (!(rbase + 8 * (q + (low ? 0 : 2)) + e < g.n)) continue;
                        const int64_t row = rbase + 8 * (q + (low ? 0 : 2)) + e;
                        packed_cell(4 * q + e, state[4 * q + e],
                                    [&](float *base, int w) __attribute__((always_inline)) { return base + row * w * H + j; });
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < 3; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
            return;
        }
        // the cell of row r (register index); at(base, w) is this lane's element of its row in a matrix of w * H columns
        auto cell = [&](int r, float prev, auto at) __attribute__((always_inline)) {
            if (LSTM) {
                const float gi = sigmoidf_(acc[0][r] + bsum[0]);
                const float gf = sigmoidf_(acc[1][r] + bsum[1]);
                const float gg = tanhf_(acc[2][r] + bsum[2]);
                const float go = sigmoidf_(acc[3][r] + bsum[LSTM ? 3 : 0]);
                const float cn = gf * prev + gi * gg;
                *at(g.c_out, 1) = cn;
                *at(g.h_out, 1) = go * tanhf_(cn);
                if (g.saved) {
                    float *sv = at(g.saved, 4);
                    sv[0] = gi;
                    sv[H] = gf;
                    sv[2 * H] = gg;
                    sv[3 * H] = go;
                }
            } else {
                const float gr = sigmoidf_(acc[0][r] + bsum[0]);
                const float gz = sigmoidf_(acc[1][r] + bsum[1]);
                const float ghn = acc[2][r] + bhn;
                const float gn = tanhf_(acc[3][r] + bsum[2] + gr * ghn);
                *at(g.h_out, 1) = (1.0f - gz) * gn + gz * prev;
                if (g.saved) {
                    float *sv = at(g.saved, 4);
                    sv[0] = gr;
                    sv[H] = gz;
                    sv[2 * H] = gn;
                    sv[3 * H] = ghn;
                }
            }
        };
        if (SPLIT && j < H && full) {
            // a whole tile: addresses from a wave-uniform part (tile, row inside it) and a constant lane part
            // (the 12-wave variants on the fp32 instructions have no registers to spare for it)
            const uint32_t hrow = uint32_t(H) * 4u;
            const int64_t tile_h = int64_t(tile) * 32 * hrow;
            const uint32_t lane_h = uint32_t(4 * kk) * hrow + uint32_t(j) * 4u, lane_s = uint32_t(16 * kk) * hrow + uint32_t(j) * 4u;
            // the tile's sixteen state values are requested together: one wait per tile instead of one per four rows
            float prev[16];
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    prev[4 * q + e] = pstate ? *reinterpret_cast<const float *>(reinterpret_cast<const char *>(pstate) + tile_h +
                                                                                uint32_t(8 * q + e) * hrow + lane_h)
                                             : 0.0f;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int64_t oh = tile_h + uint32_t(8 * q + e) * hrow;
                    cell(4 * q + e, prev[4 * q + e], [&](float *base, int w) __attribute__((always_inline)) {
                        return reinterpret_cast<float *>(reinterpret_cast<char *>(base) + w * oh + (w == 4 ? lane_s : lane_h));
                    });
                }
            }
        } else if (j < H) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                int64_t rr[4];
                float prev[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    rr[e] = min(rbase + 8 * q + e, g.n - 1);
                    prev[e] = pstate ? pstate[rr[e] * H + j] : 0.0f;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (!(full || rbase + 8 * q + e < g.n)) continue;
                    const int64_t o = rr[e] * H + j;
                    cell(4 * q + e, prev[e],
                         [&](float *base, int w) __attribute__((always_inline)) { return w == 1 ? base + o : base + rr[e] * 4 * H + j; });
                }
            }
        }
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
    };
    auto state_chunk = [&](float(&cur)[16]) __attribute__((always_inline)) {
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {  // both halves hold the wave's 16 units: the upper half takes the last eight
            float lo8 = cur[e], hi8 = cur[8 + e];
            asm volatile("" : "+v"(lo8), "+v"(hi8));
            v[e] = kk ? hi8 : lo8;
        }
        u32x4 sh, sm, sl;
        split8(v, sh, sm, sl);
        acc[2] = mfma_bf16(sl, ident, acc[2]);
        acc[2] = mfma_bf16(sm, ident, acc[2]);
        acc[2] = mfma_bf16(sh, ident, acc[2]);
    };
    auto multiply = [&](float(&cur)[16], float sc) __attribute__((always_inline)) {
        const float *bp = bp0 + kc * kBK * NC;
        if (PACK && ks && kc == kx + kh) {
            state_chunk(cur);
        } else {
            const float f = (has_xs && kc < kx) ? sc : 1.0f;
#pragma unroll
            for (int e = 0; e < 16; ++e) cur[e] *= f;
            if (PACK)
                mfma_chunk_split<2, 4>(cur, Bq + (4 * kc + 2 * kk) * NC + wn * 64 + i, NC, plane, 32, acc);
            else if (SPLIT)
                mfma_chunk_split<KG, 4>(cur, Bq + (4 * kc + 2 * kk) * NC + wn * 32 + i, NC, plane, BH, acc);
            else
                mfma_chunk_map<KG, KG - 1, G>(cur, bp, NC, BH, acc, NoPrefetch());
        }
        ++kc;
        if (!LSTM && kc == kx) {  // GRU: the x part of the n gate is complete; the h part starts from zero
            acc[3] = acc[2];
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[2][r] = 0.0f;
        }
        if (kc == kch) {
            epilogue();
            kc = 0;
            tile += stride;
        }
    };
    // steady state (unconditional loads, exact waits), then the last chunks: see gemm_rows_resident_kernel
    const int my_tiles = first < ntiles ? (ntiles - first + stride - 1) / stride : 0;
    const int steady = max(my_tiles * kch - (RING - 1), 0) / RING;
    for (int it = 0; it < steady; ++it) {
#pragma unroll
        for (int r = 0; r < RING; ++r) {
            issue_always(buf[(r + RING - 1) % RING], bsc[(r + RING - 1) % RING]);
            __builtin_amdgcn_sched_barrier(0);
            multiply(buf[r], bsc[r]);
        }
    }
    while (tile < ntiles) {
#pragma unroll
        for (int r = 0; r < RING; ++r) {
            if (tile < ntiles) {
                const float sc = bsc[r];
                issue(buf[(r + RING - 1) % RING], bsc[(r + RING - 1) % RING]);
                __builtin_amdgcn_sched_barrier(0);
                multiply(buf[r], sc);
            }
        }
    }
}

template <bool LSTM, int WN, int WAVES, bool SPLIT, bool PACK = false>
bool rnn_fused_resident_launch(const RnnArgs &g, hipStream_t s)
{
    constexpr int KG = LSTM ? 4 : 3;
    constexpr int WM = WAVES / WN;
    constexpr int UW = PACK ? 16 : 32;
    if (g.d_in % kBK != 0 || g.H % kBK != 0 || g.d_in % 4 != 0) return false;
    if (PACK && (reinterpret_cast<uintptr_t>(g.c_prev) & 15) != 0) return false;  // (the state chunk is read in 16-byte pieces)
    const size_t lds = size_t(g.d_in + g.H) * KG * UW * WN * (SPLIT ? 6 : sizeof(float));
    if (lds > kLdsBytes - 1024) return false;
    auto k = rnn_fused_resident_kernel<LSTM, WN, WAVES, SPLIT, PACK>;
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, int(lds)) != hipSuccess)
        return false;
    const int per_cu = resident_blocks(reinterpret_cast<const void *>(k), 64 * WAVES, lds);
    if (per_cu <= 0) return false;
    const int64_t ntiles = (g.n + 31) / 32;
    const unsigned gy = unsigned((g.H + UW * WN - 1) / (UW * WN));
    dim3 grid(unsigned(std::min<int64_t>((ntiles + WM - 1) / WM, std::max<int64_t>(1, int64_t(kNumCU) * per_cu / gy))), gy);
    k<<<grid, 64 * WAVES, lds, s>>>(g);
    return true;
}

constexpr int kRnnWaves = 12;  // three waves per SIMD: the kernel needs at most 168 registers

constexpr int kRnnSplitWaves = 8;  // the split variant holds three planes of every fragment: two waves per SIMD
constexpr int kRnnPackWaves = 8;   // (12 waves would leave 168 registers: the epilogue then spills)

template <bool LSTM>
bool rnn_fused_resident_dispatch(const RnnArgs &g, hipStream_t s)
{
    if (dense_split_enabled()) {  // shapes whose three-plane slab does not fit stay on the fp32 instructions
        if (g.H % 128 == 0 && rnn_fused_resident_launch<LSTM, 4, kRnnSplitWaves, true>(g, s)) return true;
        if (g.H % 64 == 0 && rnn_fused_resident_launch<LSTM, 2, kRnnSplitWaves, true>(g, s)) return true;
        if (rnn_fused_resident_launch<LSTM, 1, kRnnSplitWaves, true>(g, s)) return true;
        // LSTM whose unpacked three-plane slab does not fit: 16 units per wave, two gates per tile
        if constexpr (LSTM) {
            if (g.H % 16 == 0 && rnn_fused_resident_launch<true, 1, kRnnPackWaves, true, true>(g, s)) return true;
        }
    }
    if (g.H % 128 == 0 && rnn_fused_resident_launch<LSTM, 4, kRnnWaves, false>(g, s)) return true;
    if (g.H % 64 == 0 && rnn_fused_resident_launch<LSTM, 2, kRnnWaves, false>(g, s)) return true;
    return rnn_fused_resident_launch<LSTM, 1, kRnnWaves, false>(g, s);
}

// ---- weight / bias gradient: C[K,M] = sum_rows (rs .* A)^T G ---------------------------------------------
// grid (slab_i, slab_j, chunk); a block's 4 waves split its row chunk, each keeps a 64x64 output slab
// (2x2 accumulators), and the four partial slabs are summed through LDS.  Row K of the partial holds the
// column sums of G (the bias gradient), produced by the slab_i == 0 blocks.
struct ReduceArgs {
    const float *A;
    int lda;
    const float *row_scale;
    const float *G;
    int ldg;
    int64_t n;
    int K, M;
    int64_t rows_per_chunk;
    float *partial;  // [chunks, K+1, M]
    int chunks;
    int accumulate;  // add to the partial slabs instead of overwriting them (later timesteps of a window)
};

// One trip of a wave on the bf16 matrix cores: the lane's eight values per operand are eight rows of the trip
// (the contraction runs over rows), each operand is split into its three bfloat16 planes and the six products of
// relative size 2^-16 and above are accumulated, smallest first (see the note on fp32 products above).
__device__ inline void reduce_trip_split(const float (&a0)[8], const float (&a1)[8], const float (&g0)[8], const float (&g1)[8],
                                         acc16 (&acc)[2][2])
{
    u32x4 A0[3], A1[3], G0[3], G1[3];
    split8(g0, G0[0], G0[1], G0[2]);
    split8(g1, G1[0], G1[1], G1[2]);
    split8(a0, A0[0], A0[1], A0[2]);
    split8(a1, A1[0], A1[1], A1[2]);
    constexpr int order[6][2] = {{2, 0}, {1, 1}, {0, 2}, {1, 0}, {0, 1}, {0, 0}};
#pragma unroll
    for (int o = 0; o < 6; ++o) {
        const int p = order[o][0], q = order[o][1];
        acc[0][0] = mfma_bf16(A0[p], G0[q], acc[0][0]);
        acc[0][1] = mfma_bf16(A0[p], G1[q], acc[0][1]);
        acc[1][0] = mfma_bf16(A1[p], G0[q], acc[1][0]);
        acc[1][1] = mfma_bf16(A1[p], G1[q], acc[1][1]);
    }
}

// WIDE (outputs of four or more 64x64 slabs): the block's four waves take four different slabs (2 x 2, or 1 x 4 when
// K <= 64) over the SAME rows instead of sharing one slab over different rows.  A row of A and of G is then fetched by
// a quarter as many blocks -- with one slab per block every block re-read its 64 + 64 columns of every row, and on
// outputs of 16 slabs (128 x 512: an LSTM's gate weights) the counters showed 2.6 times the algorithmic bytes coming
// from HBM -- and no partial slabs have to be combined at the end.
template <bool HAS_RS, bool SPLIT, bool WIDE>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) gemm_reduce_kernel(ReduceArgs g)
{
    // wave w finishes accumulator tile w of the 2x2: the other waves park their share of it here (two tiles at
    // a time, to keep the block's LDS at 25 KB)
    // (wide mode with shared splitting uses the same storage for its staged planes: 3 buffers x 4 pieces x 3 planes x
    // 64 columns x 2 half-waves of 16-byte records = 72 KB; two blocks per compute unit still fit)
    constexpr int kRedFloats = 2 * 3 * 32 * 33, kBredFloats = 4 * 64;
    constexpr int kStageRecords = 3 * 4 * 3 * 64 * 2;
    constexpr size_t kSharedBytes = (SPLIT && WIDE) ? size_t(kStageRecords) * 16 : size_t(kRedFloats + kBredFloats) * 4;
    __shared__ __align__(16) unsigned char smem[kSharedBytes];
    float(*red)[3][32 * 33] = reinterpret_cast<float(*)[3][32 * 33]>(smem);
    float(*bred)[64] = reinterpret_cast<float(*)[64]>(smem + size_t(kRedFloats) * 4);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int i = lane & 31, kk = lane >> 5;
    // 1-D grid; consecutive block ids go round the 8 XCDs, so id % 8 picks the XCD.  All slabs of one row chunk
    // are given to the same XCD (and to neighbouring ids), so that chunk's rows are fetched from HBM once and the
    // other slabs find them in that XCD's L2.
    // WIDE: a block's slab is wx x wy wave slabs
    const int wx = WIDE ? (g.K > 64 ? 2 : 1) : 1, wy = WIDE ? 4 / wx : 1;
    const int slabs_x = (g.K + 64 * wx - 1) / (64 * wx), slabs = slabs_x * ((g.M + 64 * wy - 1) / (64 * wy));
    const int xcd = blockIdx.x % 8, qid = blockIdx.x / 8;
    const int slab = qid % slabs, chunk = (qid / slabs) * 8 + xcd;
    if (chunk >= g.chunks) return;
    const int f0 = (slab % slabs_x) * 64 * wx + (WIDE ? (w % wx) * 64 : 0);
    const int c0 = (slab / slabs_x) * 64 * wy + (WIDE ? (w / wx) * 64 : 0);
    if (WIDE && (f0 >= g.K || c0 >= g.M)) return;  // a wave slab outside the output (no barrier follows in this mode)
    // rows of a trip: wave offset + rstep * u + half-wave, u = 0 .. 7; a block's trip covers `trip` rows
    const int woff = WIDE ? 0 : 2 * w, rstep = WIDE ? 2 : 8, trip = WIDE ? 16 : 64;
    const int64_t r_begin = int64_t(chunk) * g.rows_per_chunk;
    const int64_t r_end = max(r_begin, min(g.n, r_begin + g.rows_per_chunk));  // a chunk past the last row is empty
    acc16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;
    float bsum[2] = {0.0f, 0.0f};
    const bool fa0 = f0 + i < g.K, fa1 = f0 + 32 + i < g.K;
    const bool cb0 = c0 + i < g.M, cb1 = c0 + 32 + i < g.M;
    // Wave w takes row pairs w, w+4, ... of the chunk, kRU pairs (64 rows of the block) per trip.  Full trips
    // over full 64x64 slabs run without a branch and double-buffered: the loads of the next trip are issued
    // before the matrix instructions of the current one, and while a next trip exists they are unconditional
    // (a load that may or may not have been issued would force a wait for everything).
    constexpr int kRU = 8;
    int64_t base = r_begin;
    // Wide 2 x 2 with the block slab inside the output: the four waves need the same 16 rows of 128 columns of A and
    // of 128 columns of G, two waves each piece of 64 columns.  Each wave loads and splits ONE piece (waves 1, 3: the
    // two pieces of A; waves 0, 2: the piece of G under their own slab, so the column sums for the bias gradient
    // come out in the waves that write them), parks its three planes in LDS, and after a barrier every wave takes
    // the fragments of the A piece and the G piece of its slab from there: half the loads and half the splitting per
    // wave, and the waves cannot drift apart.  One barrier per trip and a ring of three LDS buffers: a wave that
    // writes buffer b again has passed the barriers of the two trips between, which every wave reaches only after
    // its reads of b.  The loads run two trips ahead of the arithmetic (three register sets): with one trip in
    // flight the bytes outstanding per compute unit, not the arithmetic, bounded the rate.
    bool shared_split = false;
    if constexpr (SPLIT && WIDE) {
        // (chunks of fewer than five trips take the per-wave path below: the pipeline here starts with two trips
        // in flight and its loop runs at least once)
        shared_split = wx == 2 && (slab % slabs_x + 1) * 128 <= g.K && (slab / slabs_x + 1) * 128 <= g.M && r_end - r_begin >= 5 * 16;
        if (shared_split) {
            // [buffer][piece][plane][32-column half][lane]: a lane's record sits at its lane index, so that the lanes
            // of a 128-bit LDS access cover consecutive 16-byte records (records two apart cost every access twice)
            u32x4 *stage = reinterpret_cast<u32x4 *>(smem);
            const int wu = __builtin_amdgcn_readfirstlane(w);  // (known to be the same in every lane: scalar addresses)
            const bool a_piece = (wu & 1) != 0;
            const int piece = wu >> 1, slot = a_piece ? piece : 2 + piece;
            const int pcol0 = (a_piece ? (slab % slabs_x) : (slab / slabs_x)) * 128 + 64 * piece;
            const int ld = a_piece ? g.lda : g.ldg;
            // The loads are written as instructions with the waits placed by hand.  The compiler's own wait
            // insertion loses count of loads that cross the loop's back edge: it made the first trip of every
            // iteration wait for all loads but the newest group, which left one trip in flight instead of two.
            // Addresses: a wave-uniform base (scalar registers, advanced once per trip) plus one fixed 32-bit
            // lane offset per row pair; the second 32 columns ride on the instruction's offset field.
            const float *pp = (a_piece ? g.A : g.G) + base * ld + pcol0;
            const float *sp = HAS_RS ? g.row_scale + base : nullptr;  // (every wave loads the scales: equal load counts)
            unsigned voff[kRU], soff[kRU];
#pragma unroll
            for (int u = 0; u < kRU; ++u) {
                voff[u] = (unsigned(2 * u + kk) * unsigned(ld) + unsigned(i)) * 4u;
                soff[u] = unsigned(2 * u + kk) * 4u;
            }
            // a trip's piece: [0] [1] = its two 32-column halves, [2] = row scale
            constexpr int kGroup = HAS_RS ? 3 * kRU : 2 * kRU;  // loads per trip and wave
            static_assert(2 * kGroup <= 63, "the counter of outstanding loads holds 63");
            auto load = [&](float(&t)[3][kRU]) __attribute__((always_inline)) {
#pragma unroll
                for (int u = 0; u < kRU; ++u) {
                    asm volatile("global_load_dword %0, %1, %2" : "=&v"(t[0][u]) : "v"(voff[u]), "s"(pp) : "memory");
                    asm volatile("global_load_dword %0, %1, %2 offset:128" : "=&v"(t[1][u]) : "v"(voff[u]), "s"(pp) : "memory");
                    if (HAS_RS)
                        asm volatile("global_load_dword %0, %1, %2" : "=&v"(t[2][u]) : "v"(soff[u]), "s"(sp) : "memory");
                    else
                        t[2][u] = 1.0f;
                }
                pp += int64_t(16) * ld;
                if (HAS_RS) sp += 16;
            };
            // waits until at most NEWER * kGroup loads are outstanding: the group in `t` has arrived when NEWER
            // groups were issued after it.  The values pass through the statements, so nothing that uses them can
            // be placed ahead of the wait.  Between a load and its wait the compiler takes the destination registers
            // for ready values: the control flow below is shaped so that it has no reason to copy them there (loads
            // and waits are never separated by a branch that is taken only sometimes, except the loop's back edge,
            // where the three register sets keep their roles).
            auto arrive8 = [](float(&r)[kRU]) __attribute__((always_inline)) {
                asm volatile("" : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7])::"memory");
            };
            auto wait_for = [&](float(&t)[3][kRU], auto newer) __attribute__((always_inline)) {
                constexpr int kLeft = decltype(newer)::value * kGroup;
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLeft) : "memory");
                arrive8(t[0]);
                arrive8(t[1]);
                if (HAS_RS) arrive8(t[2]);
            };
            using Newer0 = std::integral_constant<int, 0>;
            using Newer2 = std::integral_constant<int, 2>;
            const int sx = w % 2, sy = w / 2;
            auto process = [&](float(&t)[3][kRU], int buf) __attribute__((always_inline)) {
                if (HAS_RS && a_piece) {
#pragma unroll
                    for (int u = 0; u < kRU; ++u) {
                        t[0][u] *= t[2][u];
                        t[1][u] *= t[2][u];
                    }
                }
                if (!a_piece) {  // column sums of G: the bias gradient
#pragma unroll
                    for (int u = 0; u < kRU; ++u) {
                        bsum[0] += t[0][u];
                        bsum[1] += t[1][u];
                    }
                }
                u32x4 p0[3], p1[3];
                split8(t[0], p0[0], p0[1], p0[2]);
                split8(t[1], p1[0], p1[1], p1[2]);
                u32x4 *mine = stage + ((buf * 4 + slot) * 3) * 128;  // this wave's piece
#pragma unroll
                for (int pl = 0; pl < 3; ++pl) {
                    mine[pl * 128 + lane] = p0[pl];
                    mine[pl * 128 + 64 + lane] = p1[pl];
                }
                __syncthreads();
                const u32x4 *pa = stage + ((buf * 4 + sx) * 3) * 128, *pg = stage + ((buf * 4 + 2 + sy) * 3) * 128;
                u32x4 A0[3], A1[3], G0[3], G1[3];
#pragma unroll
                for (int pl = 0; pl < 3; ++pl) {
                    A0[pl] = pa[pl * 128 + lane];
                    A1[pl] = pa[pl * 128 + 64 + lane];
                    G0[pl] = pg[pl * 128 + lane];
                    G1[pl] = pg[pl * 128 + 64 + lane];
                }
                constexpr int order[6][2] = {{2, 0}, {1, 1}, {0, 2}, {1, 0}, {0, 1}, {0, 0}};
#pragma unroll
                for (int o = 0; o < 6; ++o) {
                    const int p = order[o][0], q = order[o][1];
                    acc[0][0] = mfma_bf16(A0[p], G0[q], acc[0][0]);
                    acc[0][1] = mfma_bf16(A0[p], G1[q], acc[0][1]);
                    acc[1][0] = mfma_bf16(A1[p], G0[q], acc[1][0]);
                    acc[1][1] = mfma_bf16(A1[p], G1[q], acc[1][1]);
                }
            };
            const int trips = int((r_end - r_begin) / 16);  // at least 5
            float ta[3][kRU], tb[3][kRU], tc[3][kRU];
            int t = 0;
            load(ta);
            load(tb);
            // invariant at the top: trips t and t+1 are loaded (ta, tb) and at least three more trips follow them
            do {
                load(tc);
                wait_for(ta, Newer2());
                process(ta, 0);
                load(ta);
                wait_for(tb, Newer2());
                process(tb, 1);
                load(tb);
                wait_for(tc, Newer2());
                process(tc, 2);
                t += 3;
            } while (t + 5 <= trips);
            // two to four trips are left, the first two of them loaded: they wait for everything outstanding
            const int left = trips - t;
            wait_for(ta, Newer0());
            wait_for(tb, Newer0());
            process(ta, 0);
            process(tb, 1);
            if (left > 2) {
                load(tc);
                wait_for(tc, Newer0());
                process(tc, 2);
            }
            if (left > 3) {
                load(ta);
                wait_for(ta, Newer0());
                process(ta, 0);
            }
            base += int64_t(trips) * 16;
        }
    }
    if (!shared_split && f0 + 64 <= g.K && c0 + 64 <= g.M) {
        // wave-uniform row pointers plus one fixed 32-bit lane offset per operand: the addresses of a trip cost
        // scalar arithmetic only
        const int wu = __builtin_amdgcn_readfirstlane(woff);
        const float *ap = g.A + (base + wu) * g.lda + f0;
        const float *gp = g.G + (base + wu) * g.ldg + c0;
        const float *sp = HAS_RS ? g.row_scale + base + wu : nullptr;
        const unsigned aoff = unsigned(kk) * unsigned(g.lda) + i, goff = unsigned(kk) * unsigned(g.ldg) + i;
        // a trip's operands: [0] [1] = the two 32-column halves of the A rows, [2] [3] = of the G rows, [4] = row scale
        auto load = [&](float(&t)[5][kRU]) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < kRU; ++u) {
                const float *au = ap + int64_t(rstep * u) * g.lda, *gu = gp + int64_t(rstep * u) * g.ldg;
                t[0][u] = au[aoff];
                t[1][u] = au[aoff + 32];
                t[2][u] = gu[goff];
                t[3][u] = gu[goff + 32];
                t[4][u] = HAS_RS ? sp[rstep * u + kk] : 1.0f;
            }
            ap += int64_t(trip) * g.lda;
            gp += int64_t(trip) * g.ldg;
            if (HAS_RS) sp += trip;
        };
        auto multiply = [&](float(&t)[5][kRU]) __attribute__((always_inline)) {
            if (SPLIT) {
                static_assert(kRU == 8, "a trip is one depth-16 matrix instruction per tile: eight rows per lane");
                if (HAS_RS) {
#pragma unroll
                    for (int u = 0; u < kRU; ++u) {
                        t[0][u] *= t[4][u];
                        t[1][u] *= t[4][u];
                    }
                }
#pragma unroll
                for (int u = 0; u < kRU; ++u) {
                    bsum[0] += t[2][u];
                    bsum[1] += t[3][u];
                }
                reduce_trip_split(t[0], t[1], t[2], t[3], acc);
                return;
            }
#pragma unroll
            for (int u = 0; u < kRU; ++u) {
                const float a0 = HAS_RS ? t[0][u] * t[4][u] : t[0][u], a1 = HAS_RS ? t[1][u] * t[4][u] : t[1][u];
                acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, t[2][u], acc[0][0], 0, 0, 0);
                acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, t[3][u], acc[0][1], 0, 0, 0);
                acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, t[2][u], acc[1][0], 0, 0, 0);
                acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, t[3][u], acc[1][1], 0, 0, 0);
                bsum[0] += t[2][u];
                bsum[1] += t[3][u];
            }
        };
        const int trips = int((r_end - r_begin) / trip);
        float ta[5][kRU], tb[5][kRU];
        int t = 0;
        if (trips > 0) load(ta);
        // WIDE: the four waves read the same rows (two of them the same columns of A, two the same columns of G).  While
        // the whole block slab lies inside the output all four run this loop with the same trip count, and a barrier
        // every other trip keeps them within two trips of each other, so that the second request for a line finds it in
        // the compute unit's cache instead of going out again.
        const bool lockstep = WIDE && (slab % slabs_x + 1) * 64 * wx <= g.K && (slab / slabs_x + 1) * 64 * wy <= g.M;
        for (; t + 2 < trips; t += 2) {
            if (lockstep) __syncthreads();
            load(tb);
            __builtin_amdgcn_sched_barrier(0);  // the loads go out ahead of the arithmetic
            multiply(ta);
            load(ta);
            __builtin_amdgcn_sched_barrier(0);
            multiply(tb);
        }
        if (t + 1 < trips) {
            load(tb);
            __builtin_amdgcn_sched_barrier(0);
            multiply(ta);
            multiply(tb);
        } else if (t < trips) {
            multiply(ta);
        }
        base += int64_t(trips) * trip;
    }
    // ragged slabs and the last rows of the chunk: guarded loads
    for (int64_t r0 = base + woff + kk; r0 < r_end + kk; r0 += trip) {
        // (the bound keeps both half-waves in step: a half that runs past r_end loads zeros)
        float a0[kRU], a1[kRU], b0[kRU], b1[kRU];
#pragma unroll
        for (int u = 0; u < kRU; ++u) {
            const int64_t r = r0 + rstep * u;
            a0[u] = a1[u] = b0[u] = b1[u] = 0.0f;
            if (r < r_end) {
                const float sc = HAS_RS ? g.row_scale[r] : 1.0f;
                const float *ap = g.A + r * g.lda + f0 + i;
                const float *gp = g.G + r * g.ldg + c0 + i;
                if (fa0) a0[u] = ap[0] * sc;
                if (fa1) a1[u] = ap[32] * sc;
                if (cb0) b0[u] = gp[0];
                if (cb1) b1[u] = gp[32];
            }
        }
        if (SPLIT) {
#pragma unroll
            for (int u = 0; u < kRU; ++u) {
                bsum[0] += b0[u];
                bsum[1] += b1[u];
            }
            reduce_trip_split(a0, a1, b0, b1, acc);
            continue;
        }
#pragma unroll
        for (int u = 0; u < kRU; ++u) {
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[u], b0[u], acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[u], b1[u], acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[u], b0[u], acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[u], b1[u], acc[1][1], 0, 0, 0);
            bsum[0] += b0[u];
            bsum[1] += b1[u];
        }
    }
    float *out = g.partial + int64_t(chunk) * (g.K + 1) * g.M;
    if (WIDE) {
        // every wave owns its four tiles: straight to the partial slab, four rows at a time
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int cc = c0 + 32 * b + i;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int fr = f0 + 32 * a + 8 * q + 4 * kk + e;
                        if (fr < g.K && cc < g.M) {
                            float *o = out + int64_t(fr) * g.M + cc;
                            *o = g.accumulate ? *o + acc[a][b][4 * q + e] : acc[a][b][4 * q + e];
                        }
                    }
                }
            }
        if (f0 == 0) {  // the bias gradient: column sums of G, from the waves of the first row of slabs
            const float s0 = bsum[0] + __shfl_xor(bsum[0], 32), s1 = bsum[1] + __shfl_xor(bsum[1], 32);
            if (kk == 0) {
                float *o = out + int64_t(g.K) * g.M + c0 + i;
                if (c0 + i < g.M) o[0] = g.accumulate ? o[0] + s0 : s0;
                if (c0 + 32 + i < g.M) o[32] = g.accumulate ? o[32] + s1 : s1;
            }
        }
        return;
    }
    // Combine the four waves.  Tile (a, b) is finished by wave 2a+b: the other three park their share in LDS
    // (slot = their rank among the other waves) and the owner adds the four shares in wave order, then adds
    // the result to the partial slab (or overwrites it).  Tiles (0, *) go first, then tiles (1, *).
    {
        const float s0 = bsum[0] + __shfl_xor(bsum[0], 32), s1 = bsum[1] + __shfl_xor(bsum[1], 32);
        if (kk == 0) {
            bred[w][i] = s0;
            bred[w][32 + i] = s1;
        }
    }
    auto park = [&](const acc16 &t, int owner) __attribute__((always_inline)) {
        float *dst = red[owner & 1][w < owner ? w : w - 1];
#pragma unroll
        for (int r = 0; r < 16; ++r) dst[(8 * (r / 4) + 4 * kk + (r % 4)) * 33 + i] = t[r];
    };
    auto finish = [&](const acc16 &mine, int a, int b) __attribute__((always_inline)) {
        const int cc = c0 + 32 * b + i;
        const int owner = 2 * a + b;
#pragma unroll
        for (int q = 0; q < 4; ++q) {  // four rows at a time keeps the register count of the tail low
            float old[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (g.accumulate) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int fr = f0 + 32 * a + 8 * q + 4 * kk + e;
                    if (fr < g.K && cc < g.M) old[e] = out[int64_t(fr) * g.M + cc];
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int lr = 8 * q + 4 * kk + e;
                float v = 0.0f;
#pragma unroll
                for (int ww = 0; ww < 4; ++ww)  // shares in wave order: a fixed summation order
                    v += ww == owner ? mine[4 * q + e] : red[b][ww < owner ? ww : ww - 1][lr * 33 + i];
                const int fr = f0 + 32 * a + lr;
                if (fr < g.K && cc < g.M) out[int64_t(fr) * g.M + cc] = old[e] + v;
            }
        }
    };
    if (w != 0) park(acc[0][0], 0);
    if (w != 1) park(acc[0][1], 1);
    __syncthreads();
    if (w == 0) finish(acc[0][0], 0, 0);
    if (w == 1) finish(acc[0][1], 0, 1);
    __syncthreads();
    if (w != 2) park(acc[1][0], 2);
    if (w != 3) park(acc[1][1], 3);
    __syncthreads();
    if (w == 2) finish(acc[1][0], 1, 0);
    if (w == 3) finish(acc[1][1], 1, 1);
    if (w == 0 && f0 == 0 && c0 + lane < g.M) {
        float *o = out + int64_t(g.K) * g.M + c0 + lane;
        const float v = ((bred[0][lane] + bred[1][lane]) + bred[2][lane]) + bred[3][lane];
        *o = g.accumulate ? *o + v : v;
    }
}

// dst_w[K*M] += sum_c partial[c][0..K*M);  dst_b[M] += sum_c partial[c][K*M ..)
// A block owns 64 consecutive outputs; its 16 waves split the chunks (four independent sums each, so that the
// loads of a wave overlap), then wave 0 adds the 16 sums in wave order: a fixed summation order.
constexpr int kPartialWaves = 16;

__global__ void __launch_bounds__(64 * kPartialWaves)
reduce_partials_kernel(const float *partial, int chunks, int K, int M, float *dst_w, float *dst_b)
{
    __shared__ float red[kPartialWaves][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int total = (K + 1) * M;
    const int idx = blockIdx.x * 64 + lane;
    float s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (idx < total) {
        int c = w;
        for (; c + 3 * kPartialWaves < chunks; c += 4 * kPartialWaves) {
#pragma unroll
            for (int u = 0; u < 4; ++u) s[u] += partial[int64_t(c + u * kPartialWaves) * total + idx];
        }
        for (int u = 0; c < chunks; c += kPartialWaves, ++u) s[u] += partial[int64_t(c) * total + idx];
    }
    red[w][lane] = (s[0] + s[1]) + (s[2] + s[3]);
    __syncthreads();
    if (w != 0 || idx >= total) return;
    float v = red[0][lane];
#pragma unroll
    for (int ww = 1; ww < kPartialWaves; ++ww) v += red[ww][lane];
    if (idx < K * M)
        dst_w[idx] += v;
    else if (dst_b)
        dst_b[idx - K * M] += v;
}

// ---- column sums of a tall matrix (bias gradient of a layer whose linear map runs before its aggregation) -------
// Block b adds the rows b, b + blocks, ... (thread j of 256 takes the columns j, j + 256, ...: coalesced rows); the
// second kernel adds the blocks' sums in block order: a fixed summation order.
constexpr int kColumnSumBlocks = 1024;

__global__ void __launch_bounds__(256) column_sums_partial(const float *__restrict__ G, int64_t n, int M, float *__restrict__ partial)
{
    for (int j = threadIdx.x; j < M; j += 256) {
        float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
        int64_t r = blockIdx.x;
        for (; r + 3 * int64_t(kColumnSumBlocks) < n; r += 4 * int64_t(kColumnSumBlocks)) {
            s0 += G[r * M + j];
            s1 += G[(r + kColumnSumBlocks) * M + j];
            s2 += G[(r + 2 * int64_t(kColumnSumBlocks)) * M + j];
            s3 += G[(r + 3 * int64_t(kColumnSumBlocks)) * M + j];
        }
        for (; r < n; r += kColumnSumBlocks) s0 += G[r * M + j];
        partial[int64_t(blockIdx.x) * M + j] = (s0 + s1) + (s2 + s3);
    }
}

__global__ void __launch_bounds__(256) column_sums_finish(const float *__restrict__ partial, int M, float *db, int accumulate)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= M) return;
    float s = 0.0f;
    for (int b = 0; b < kColumnSumBlocks; ++b) s += partial[int64_t(b) * M + j];
    db[j] = accumulate ? db[j] + s : s;
}

// ---- recurrent backward, elementwise part ------------------------------------------------------------------
// GRU : dgi = [dr, dz, dn], dgh = [dr, dz, dn .* r], dh_carry = dh .* z
// LSTM: dgi = dgh = [di, df, dg, do], dc_prev = dc_total .* f, dh_carry = 0
struct RnnBwdArgs {
    int64_t n;
    int H;
    const float *dh, *dc;  // gradient w.r.t. h_t (and c_t; may be null = 0)
    const float *saved;    // [n, 4H]
    const float *h_prev, *c_prev, *c_new;  // null = zero state
    float *dgi, *dgh;      // [n, K*H]
    float *dh_carry;       // [n, H]
    float *dc_prev;        // [n, H] (LSTM)
};

template <bool LSTM>
__global__ void rnn_backward_elem_kernel(RnnBwdArgs g)
{
    const int64_t idx = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (idx >= g.n * g.H) return;
    const int64_t r = idx / g.H;
    const int j = int(idx - r * g.H);
    const int H = g.H;
    const float *sv = g.saved + r * 4 * H + j;
    const float dh = g.dh[idx];
    if (LSTM) {
        const float gi = sv[0], gf = sv[H], gg = sv[2 * H], go = sv[3 * H];
        const float tc = tanhf_(g.c_new[idx]);
        const float dcc = (g.dc ? g.dc[idx] : 0.0f) + dh * go * (1.0f - tc * tc);
        const float cp = g.c_prev ? g.c_prev[idx] : 0.0f;
        float *o = g.dgi + r * 4 * H + j;
        o[0] = dcc * gg * gi * (1.0f - gi);
        o[H] = dcc * cp * gf * (1.0f - gf);
        o[2 * H] = dcc * gi * (1.0f - gg * gg);
        o[3 * H] = dh * tc * go * (1.0f - go);
        g.dc_prev[idx] = dcc * gf;
    } else {
        const float gr = sv[0], gz = sv[H], gn = sv[2 * H], ghn = sv[3 * H];
        const float hp = g.h_prev ? g.h_prev[idx] : 0.0f;
        const float dn = dh * (1.0f - gz) * (1.0f - gn * gn);
        const float dz = dh * (hp - gn) * gz * (1.0f - gz);
        const float dr = dn * ghn * gr * (1.0f - gr);
        float *oi = g.dgi + r * 3 * H + j;
        float *oh = g.dgh + r * 3 * H + j;
        oi[0] = dr;
        oi[H] = dz;
        oi[2 * H] = dn;
        oh[0] = dr;
        oh[H] = dz;
        oh[2 * H] = dn * gr;
        g.dh_carry[idx] = dh * gz;
    }
}

// ---- loss ----------------------------------------------------------------------------------------------------
constexpr int kLossBlocks = 1024;

// Partial sums of squared errors, one per block, in a fixed order.  VEC = 4 reads 16 bytes per lane (needs aligned
// pointers); four independent loads per lane are in flight.
template <int VEC>
__global__ void __launch_bounds__(256) mse_partial_kernel(const float *h, const float *y, int64_t total, float *partial)
{
    __shared__ float red[256];
    constexpr int U = 4;
    const int64_t nv = total / VEC;  // whole vectors; the tail is taken by block 0 below
    const int64_t stride = int64_t(gridDim.x) * 256;
    float s[U] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int64_t i0 = blockIdx.x * int64_t(256) + threadIdx.x; i0 < nv; i0 += U * stride) {
        float a[U][VEC], b[U][VEC];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = min(i0 + u * stride, nv - 1);
            if (VEC == 4) {
                const float4 va = reinterpret_cast<const float4 *>(h)[i], vb = reinterpret_cast<const float4 *>(y)[i];
                a[u][0] = va.x, a[u][1 % VEC] = va.y, a[u][2 % VEC] = va.z, a[u][3 % VEC] = va.w;
                b[u][0] = vb.x, b[u][1 % VEC] = vb.y, b[u][2 % VEC] = vb.z, b[u][3 % VEC] = vb.w;
            } else {
                a[u][0] = h[i];
                b[u][0] = y[i];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (i0 + u * stride < nv) {
#pragma unroll
                for (int k = 0; k < VEC; ++k) {
                    const float e = a[u][k] - b[u][k];
                    s[u] += e * e;
                }
            }
        }
    }
    float t = (s[0] + s[1]) + (s[2] + s[3]);
    if (blockIdx.x == 0 && threadIdx.x == 0)
        for (int64_t i = nv * VEC; i < total; ++i) {
            const float e = h[i] - y[i];
            t += e * e;
        }
    red[threadIdx.x] = t;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

__global__ void __launch_bounds__(256) mse_final_kernel(const float *partial, int nparts, int64_t total, float *loss)
{
    __shared__ float red[256];
    float t = 0.0f;
    for (int i = threadIdx.x; i < nparts; i += 256) t += partial[i];
    red[threadIdx.x] = t;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = total > 0 ? red[0] / float(total) : 0.0f;
}

// the loss covers the first `counted` elements; the gradient of the others (up to `total`) is zero
__global__ void mse_grad_kernel(const float *h, const float *y, int64_t counted, int64_t total, float *dh)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i < total) dh[i] = i < counted ? 2.0f * (h[i] - y[i]) / float(counted) : 0.0f;
}

__global__ void sgd_kernel(float *p, const float *g, int64_t n, float lr)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i < n) p[i] -= lr * g[i];
}

__global__ void fill_f32_kernel(float *p, int64_t n, float v)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i < n) p[i] = v;
}

}  // namespace

int launch_gemm_rows(const void *A, int a_bf16, int64_t n, int32_t K, int32_t M, const float *row_scale, const float *W,
                     int w_transposed, int32_t ldw, const float *bias, int relu, const float *add, const float *mask,
                     float *out, hipStream_t s)
{
    if (n <= 0) return 0;
    GemmArgs g{A, n, K, M, K, row_scale, W, ldw, w_transposed, bias, relu, mask, add, out};
    // Deep products (K = 512: the gate gradients of an LSTM times W^T) whose three-plane slab fits for half of K only:
    // two passes over the halves of K, the second adding to the first (out = A1 W1 + add, then out = A2 W2 + out).
    // Without bias and ReLU the epilogue order (add, then mask) makes the two passes equal to the single product.
    constexpr size_t kSlabMax = kLdsBytes - 1024;
    if (dense_split_enabled() && !bias && !relu && K % 64 == 0 && size_t(K) * 64 * 6 > kSlabMax && size_t(K / 2) * 64 * 6 <= kSlabMax &&
        M > 64) {
        const int half = K / 2;
        const char *A2 = static_cast<const char *>(A) + size_t(half) * (a_bf16 ? 2 : 4);
        const float *W2 = w_transposed ? W + half : W + int64_t(half) * ldw;
        GemmArgs g1{A, n, half, M, K, row_scale, W, ldw, w_transposed, nullptr, 0, nullptr, add, out};
        GemmArgs g2{A2, n, half, M, K, row_scale, W2, ldw, w_transposed, nullptr, 0, mask, out, out};
        if (gemm_rows_resident_dispatch(g1, a_bf16, s)) {
            if (gemm_rows_resident_dispatch(g2, a_bf16, s)) return 0;
            return -1;  // cannot happen: the second pass has the shape of the first
        }
    }
    // preferred: weight slab resident in LDS, as wide as fits
    if (gemm_rows_resident_dispatch(g, a_bf16, s)) return 0;
    // very deep products: stage the weights 32 k values at a time
    if (M <= 32)
        gemm_rows_launch<1, 4, 1>(g, a_bf16, s);
    else if (M <= 64)
        gemm_rows_launch<2, 4, 1>(g, a_bf16, s);
    else if (M <= 128)
        gemm_rows_launch<4, 4, 1>(g, a_bf16, s);
    else
        gemm_rows_launch<4, 2, 2>(g, a_bf16, s);  // 256 columns per block; wider outputs tile over blockIdx.y
    return 0;
}

void launch_rnn_fused(int lstm, const float *x, const float *x_scale, int64_t n, int32_t d_in, int32_t H, const float *h_prev,
                      const float *h_carry, const float *c_prev, const float *W_i, const float *W_h, const float *b_i,
                      const float *b_h, float *h_out, float *c_out, float *saved, hipStream_t s)
{
    if (n <= 0) return;
    RnnArgs g{x, n, d_in, H, h_prev, c_prev, x_scale, h_carry, W_i, W_h, b_i, b_h, h_out, c_out, saved};
    if (lstm ? rnn_fused_resident_dispatch<true>(g, s) : rnn_fused_resident_dispatch<false>(g, s)) return;
#define REINC_RNN_LAUNCH(WM, WN)                                                                    \
    do {                                                                                            \
        dim3 grid(unsigned((n + 32 * WM - 1) / (32 * WM)), unsigned((H + 32 * WN - 1) / (32 * WN))); \
        if (lstm)                                                                                   \
            rnn_fused_kernel<true, WM, WN><<<grid, 256, 0, s>>>(g);                                 \
        else                                                                                        \
            rnn_fused_kernel<false, WM, WN><<<grid, 256, 0, s>>>(g);                                \
    } while (0)
    if (H <= 32)
        REINC_RNN_LAUNCH(4, 1);
    else if (H <= 64)
        REINC_RNN_LAUNCH(2, 2);
    else
        REINC_RNN_LAUNCH(1, 4);
#undef REINC_RNN_LAUNCH
}

// Outputs of four or more 64x64 slabs take the wide mode (a block = four slabs over the same rows).
bool reduce_wide(int32_t K, int32_t M) { return ((K + 63) / 64) * ((M + 63) / 64) >= 4; }

int reduce_block_slabs(int32_t K, int32_t M)
{
    if (!reduce_wide(K, M)) return ((K + 63) / 64) * ((M + 63) / 64);
    const int wx = K > 64 ? 2 : 1, wy = 4 / wx;
    return ((K + 64 * wx - 1) / (64 * wx)) * ((M + 64 * wy - 1) / (64 * wy));
}

int reduce_chunks(int64_t n, int32_t K, int32_t M)
{
    // as many blocks as are resident at once (registers and LDS decide how many fit a compute unit), at least
    // 256 rows each
    static const int per_cu = [] {
        auto fit = [](const void *k) { return resident_blocks(k, 256, 0); };
        const bool split = dense_split_enabled();
        int m = 64;
        for (const void *k : {reinterpret_cast<const void *>(split ? gemm_reduce_kernel<false, true, false> : gemm_reduce_kernel<false, false, false>),
                              reinterpret_cast<const void *>(split ? gemm_reduce_kernel<true, true, false> : gemm_reduce_kernel<true, false, false>),
                              reinterpret_cast<const void *>(split ? gemm_reduce_kernel<false, true, true> : gemm_reduce_kernel<false, false, true>),
                              reinterpret_cast<const void *>(split ? gemm_reduce_kernel<true, true, true> : gemm_reduce_kernel<true, false, true>)})
            m = std::min(m, fit(k));
        return std::max(1, m);
    }();
    const int64_t slabs = reduce_block_slabs(K, M);
    int64_t chunks = std::max<int64_t>(1, int64_t(kNumCU) * per_cu / slabs);
    if (chunks >= 8) chunks &= ~int64_t(7);  // the grid is padded to whole groups of 8 chunks (one per XCD): stay resident
    chunks = std::min<int64_t>(chunks, (n + 255) / 256);
    return int(std::max<int64_t>(chunks, 1));
}

uint64_t reduce_partial_bytes(int64_t n, int32_t K, int32_t M)
{
    return uint64_t(reduce_chunks(n, K, M)) * uint64_t(K + 1) * M * 4;
}

void launch_gemm_reduce(const float *A, int32_t lda, const float *row_scale, const float *G, int32_t ldg, int64_t n,
                        int64_t n_geom, int32_t K, int32_t M, float *partial, int accumulate, hipStream_t s)
{
    if (n <= 0 || n_geom < n) return;
    // the chunk geometry (how many slabs, how many rows each) belongs to n_geom rows: calls with fewer rows fill
    // the same slabs (their last chunks see no rows and contribute zeros)
    const int chunks = reduce_chunks(n_geom, K, M);
    int64_t rpc = (n_geom + chunks - 1) / chunks;
    rpc = (rpc + 63) & ~int64_t(63);  // whole 64-row trips; no row pair straddles two chunks
    ReduceArgs g{A, lda, row_scale, G, ldg, n, K, M, rpc, partial, chunks, accumulate};
    const int slabs = reduce_block_slabs(K, M);
    const unsigned blocks = unsigned(slabs) * unsigned((chunks + 7) / 8) * 8u;
    const bool split = dense_split_enabled(), wide = reduce_wide(K, M);
    auto pick = [&](auto has_rs) {
        constexpr bool RS = decltype(has_rs)::value;
        if (wide) return split ? gemm_reduce_kernel<RS, true, true> : gemm_reduce_kernel<RS, false, true>;
        return split ? gemm_reduce_kernel<RS, true, false> : gemm_reduce_kernel<RS, false, false>;
    };
    if (row_scale)
        pick(std::true_type{})<<<blocks, 256, 0, s>>>(g);
    else
        pick(std::false_type{})<<<blocks, 256, 0, s>>>(g);
}

uint64_t column_sums_bytes(int32_t M) { return uint64_t(kColumnSumBlocks) * uint64_t(M) * sizeof(float); }

void launch_column_sums(const float *G, int64_t n, int32_t M, float *partial, float *db, int accumulate, hipStream_t s)
{
    if (n <= 0 || M <= 0) return;
    column_sums_partial<<<kColumnSumBlocks, 256, 0, s>>>(G, n, M, partial);
    column_sums_finish<<<(M + 255) / 256, 256, 0, s>>>(partial, M, db, accumulate);
}

void launch_reduce_partials(const float *partial, int64_t n, int32_t K, int32_t M, float *dW, float *db, hipStream_t s)
{
    if (n <= 0) return;
    const int total = (K + 1) * M;
    reduce_partials_kernel<<<(total + 63) / 64, 64 * kPartialWaves, 0, s>>>(partial, reduce_chunks(n, K, M), K, M, dW, db);
}

void launch_rnn_backward_elem(int lstm, int64_t n, int32_t H, const float *dh, const float *dc, const float *saved,
                              const float *h_prev, const float *c_prev, const float *c_new, float *dgi, float *dgh,
                              float *dh_carry, float *dc_prev, hipStream_t s)
{
    const int64_t total = n * H;
    if (total <= 0) return;
    RnnBwdArgs g{n, H, dh, dc, saved, h_prev, c_prev, c_new, dgi, dgh, dh_carry, dc_prev};
    const unsigned blocks = unsigned((total + 255) / 256);
    if (lstm)
        rnn_backward_elem_kernel<true><<<blocks, 256, 0, s>>>(g);
    else
        rnn_backward_elem_kernel<false><<<blocks, 256, 0, s>>>(g);
}

uint64_t loss_partial_bytes() { return kLossBlocks * sizeof(float); }

void launch_mse(const float *h, const float *y, int64_t total, float *partial, float *loss, hipStream_t s)
{
    if (((reinterpret_cast<uintptr_t>(h) | reinterpret_cast<uintptr_t>(y)) & 15) == 0)
        mse_partial_kernel<4><<<kLossBlocks, 256, 0, s>>>(h, y, total, partial);
    else
        mse_partial_kernel<1><<<kLossBlocks, 256, 0, s>>>(h, y, total, partial);
    mse_final_kernel<<<1, 256, 0, s>>>(partial, kLossBlocks, total, loss);
}

void launch_mse_grad(const float *h, const float *y, int64_t counted, int64_t total, float *dh, hipStream_t s)
{
    if (total > 0) mse_grad_kernel<<<unsigned((total + 255) / 256), 256, 0, s>>>(h, y, counted, total, dh);
}

void launch_sgd(float *params, const float *grads, int64_t n, float lr, hipStream_t s)
{
    if (n > 0) sgd_kernel<<<unsigned((n + 255) / 256), 256, 0, s>>>(params, grads, n, lr);
}

void launch_fill_f32(float *p, int64_t n, float v, hipStream_t s)
{
    if (n > 0) fill_f32_kernel<<<unsigned((n + 255) / 256), 256, 0, s>>>(p, n, v);
}

}  // namespace reinc
