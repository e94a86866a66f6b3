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

namespace reinc {

namespace {

typedef float acc16 __attribute__((ext_vector_type(16)));

#ifndef REINC_GEMM64_NT
#define REINC_GEMM64_NT 1  // accumulator tiles per wave for outputs of 33..64 columns (1: two waves share a row tile)
#endif

constexpr int kBK = 32;  // k values staged per LDS chunk

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

// 16 k-steps against B fragments in LDS.  bp points at this lane's column of the first of its 16 B rows;
// tile t of NT sits at column offset tile_stride * t.  Fragments are read four steps ahead of their use so
// that the matrix cores never wait for an LDS round trip.
template <int NT, class Prefetch>
__device__ inline void mfma_chunk(const float (&a)[16], const float *bp, int ld, int tile_stride, acc16 (&acc)[NT],
                                  Prefetch prefetch)
{
    // groups of G steps: all B fragments of a group are read from LDS first, then its matrix instructions run
    // back to back (the scheduling barriers keep the compiler from sinking each read next to its use, which
    // would expose one LDS round trip per step)
    constexpr int G = 8;
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
            for (int t = 0; t < NT; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[G * q + s], b[s][t], acc[t], 0, 0, 0);
        if (q == 0) prefetch();
        __builtin_amdgcn_sched_barrier(0);
    }
}

struct NoPrefetch {
    __device__ void operator()() const {}
};

// Same product with the whole weight slab [K, 32*NT] resident in LDS: it is staged once per block, after which
// every wave streams its own 32-row tiles without any barrier.  The k chunks of all of a wave's tiles form one
// stream; a ring of three register buffers keeps the loads two chunks (8 KB per wave) ahead of the matrix
// cores, across tile boundaries and epilogues.  Needs K % 32 == 0 and 16-byte aligned rows; the row scale is
// applied to the finished sums.
template <int NT, int WN, bool BF16>
__global__ void __launch_bounds__(256, NT == 1 ? 4 : (NT == 2 ? 3 : 2)) gemm_rows_resident_kernel(GemmArgs g)
{
    // 4 waves = (4 / WN) row tiles x WN column groups of 32*NT columns; the slab holds all 32*NT*WN columns
    extern __shared__ float Bs[];
    constexpr int BN = 32 * NT * WN;
    constexpr int WR = 4 / WN;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int wn = w % WN, wr = w / WN;
    const int i = lane & 31, kk = lane >> 5;
    const int col0 = blockIdx.y * BN;
    for (int k0 = 0; k0 < g.K; k0 += kBK)
        stage_b(Bs + k0 * BN, BN, BN, g.W, g.ldw, g.wT != 0, k0, g.K, [&](int c) { return col0 + c < g.M ? col0 + c : -1; });
    __syncthreads();
    const int64_t ntiles = (g.n + 31) / 32;
    const int64_t first = int64_t(blockIdx.x) * WR + wr, stride = int64_t(gridDim.x) * WR;
    if (first >= ntiles) return;
    const int kch = g.K / kBK;
    const int64_t total = ((ntiles - first + stride - 1) / stride) * kch;
    const float *bp0 = Bs + (16 * kk) * BN + wn * 32 * NT + i;
    const int wcol0 = col0 + wn * 32 * NT;

    // load cursor
    int64_t ltile = first, issued = 0;
    int lk = 0;
    int64_t lrow = min(ltile * 32 + i, g.n - 1);
    auto issue = [&](float(&buf)[16]) {
        if (issued < total) {
            load_a16_fast<BF16>(g.A, lrow, g.lda, lk * kBK, buf);
            ++issued;
            if (++lk == kch) {
                lk = 0;
                ltile += stride;
                lrow = min(ltile * 32 + i, g.n - 1);
            }
        }
    };
    // compute cursor
    int64_t tile = first;
    int kc = 0;
    acc16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;

    auto epilogue = [&]() {  // rows rbase + 8*(r/4) + r%4 of the finished tile
        const int64_t rbase = tile * 32 + 4 * kk;
        const bool full = tile * 32 + 32 <= g.n;
        float rs[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) rs[r] = 1.0f;
        if (g.row_scale) {
#pragma unroll
            for (int r = 0; r < 16; ++r) rs[r] = g.row_scale[min(rbase + 8 * (r / 4) + (r % 4), g.n - 1)];
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int c = wcol0 + 32 * t + i;
            if (c < g.M) {
                const float bias = g.bias ? g.bias[c] : 0.0f;
                float v[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    v[r] = acc[t][r] * rs[r] + bias;
                    if (g.relu) v[r] = fmaxf(v[r], 0.0f);
                }
                if (g.add) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) v[r] += g.add[min(rbase + 8 * (r / 4) + (r % 4), g.n - 1) * g.M + c];
                }
                if (g.mask) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (!(g.mask[min(rbase + 8 * (r / 4) + (r % 4), g.n - 1) * g.M + c] > 0.0f)) v[r] = 0.0f;
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t rr = rbase + 8 * (r / 4) + (r % 4);
                    if (full || rr < g.n) g.out[rr * g.M + c] = v[r];
                }
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
        }
    };
    auto step = [&](float(&cur)[16], float(&nxt)[16]) {
        issue(nxt);
        __builtin_amdgcn_sched_barrier(0);  // the new loads go out before this chunk's matrix instructions
        mfma_chunk<NT>(cur, bp0 + kc * kBK * BN, BN, 32, acc, NoPrefetch());
        if (++kc == kch) {
            epilogue();
            kc = 0;
            tile += stride;
        }
    };
    float b0[16], b1[16], b2[16];
    issue(b0);
    issue(b1);
    for (int64_t p = 0; p < total; p += 3) {
        step(b0, b2);
        if (p + 1 < total) step(b1, b0);
        if (p + 2 < total) step(b2, b1);
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

template <int NT, int WN>
bool gemm_rows_resident_launch(const GemmArgs &g, int bf16, hipStream_t s)
{
    if (g.K % kBK != 0 || g.lda % 8 != 0) return false;
    constexpr int BN = 32 * NT * WN;
    const size_t lds = size_t(g.K) * BN * sizeof(float);
    if (lds > kLdsBytes - 1024) return false;
    auto k = bf16 ? gemm_rows_resident_kernel<NT, WN, true> : gemm_rows_resident_kernel<NT, WN, false>;
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, int(lds)) != hipSuccess)
        return false;
    const int per_cu = resident_blocks(reinterpret_cast<const void *>(k), 256, lds);
    if (per_cu <= 0) return false;
    const int64_t ntiles = (g.n + 31) / 32;
    const int wr = 4 / WN;
    const unsigned gy = unsigned((g.M + BN - 1) / BN);
    dim3 grid(unsigned(std::min<int64_t>((ntiles + wr - 1) / wr, std::max<int64_t>(1, int64_t(kNumCU) * per_cu / gy))), gy);
    k<<<grid, 256, lds, s>>>(g);
    return true;
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
    const float *W_i, *W_h, *b_i, *b_h;
    float *h_out, *c_out, *saved;
};

__device__ inline float sigmoidf_(float v) { return 1.0f / (1.0f + expf(-v)); }

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
            load_a16<false>(A, row, g.n, K, k0, K, vec_ok, 1.0f, a);
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
            const float gg = tanhf(acc[2][r] + bi[2] + bh[2]);
            const float go = sigmoidf_(acc[3][r] + bi[3] + bh[3]);
            const float cp = g.c_prev ? g.c_prev[o] : 0.0f;
            const float cn = gf * cp + gi * gg;
            g.c_out[o] = cn;
            g.h_out[o] = go * tanhf(cn);
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
            const float gn = tanhf(acc[2][r] + bi[2] + gr * ghn);
            const float hp = g.h_prev ? g.h_prev[o] : 0.0f;
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
// staged once per block, then 8 waves (WM row tiles x WN groups of 32 hidden units) stream row tiles without
// barriers.  Rows [0, d_in) of the slab hold W_i, rows [d_in, d_in + H) hold W_h.  Needs d_in % 64 == 0 and
// H % 64 == 0.
template <bool LSTM, int WN>
__global__ void __launch_bounds__(512) rnn_fused_resident_kernel(RnnArgs g)
{
    extern __shared__ float Bs[];
    constexpr int KG = LSTM ? 4 : 3;
    constexpr int WM = 8 / WN;
    constexpr int BH = 32 * WN;
    constexpr int NC = KG * BH;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int wm = w / WN, wn = w % WN;
    const int i = lane & 31, kk = lane >> 5;
    const int h0 = blockIdx.y * BH;
    const int H = g.H, ldw = KG * H, dpad = g.d_in;
    auto col_of = [&](int c) {
        const int gate = c / BH, j = c - gate * BH;
        return h0 + j < H ? gate * H + h0 + j : -1;
    };
    for (int k0 = 0; k0 < g.d_in; k0 += kBK) stage_b(Bs + k0 * NC, NC, NC, g.W_i, ldw, false, k0, g.d_in, col_of);
    for (int k0 = 0; k0 < H; k0 += kBK) stage_b(Bs + (dpad + k0) * NC, NC, NC, g.W_h, ldw, false, k0, H, col_of);
    __syncthreads();
    const int j = h0 + wn * 32 + i;
    float bi[KG], bh[KG];
#pragma unroll
    for (int t = 0; t < KG; ++t) {
        bi[t] = (g.b_i && j < H) ? g.b_i[t * H + j] : 0.0f;
        bh[t] = (g.b_h && j < H) ? g.b_h[t * H + j] : 0.0f;
    }
    const int64_t ntiles = (g.n + 31) / 32;
    const float *bp0 = Bs + (16 * kk) * NC + wn * 32 + i;
    float a0[16], a1[16];
    bool first = true;
    for (int64_t tile = int64_t(blockIdx.x) * WM + wm; tile < ntiles; tile += int64_t(gridDim.x) * WM) {
        const int64_t row = min(tile * 32 + i, g.n - 1);
        acc16 acc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
        if (first) {
            load_a16_fast<false>(g.x, row, g.d_in, 0, a0);
            first = false;
        }
        const int64_t next_tile = tile + int64_t(gridDim.x) * WM;
        const int64_t next_row = min(next_tile * 32 + i, g.n - 1);
        const bool has_h = g.h_prev != nullptr;
        acc16(&acc3)[3] = reinterpret_cast<acc16(&)[3]>(acc[0]);
        acc16(&acc2)[2] = reinterpret_cast<acc16(&)[2]>(acc[0]);
        acc16(&acc1)[1] = reinterpret_cast<acc16(&)[1]>(acc[3]);
        // x part: gates land in accumulators 0 .. KG-1
        for (int k0 = 0; k0 < g.d_in; k0 += 2 * kBK) {
            auto pf1 = [&] { load_a16_fast<false>(g.x, row, g.d_in, k0 + kBK, a1); };
            auto pf0 = [&] {
                if (k0 + 2 * kBK < g.d_in)
                    load_a16_fast<false>(g.x, row, g.d_in, k0 + 2 * kBK, a0);
                else if (has_h)
                    load_a16_fast<false>(g.h_prev, row, H, 0, a0);
                else if (next_tile < ntiles)
                    load_a16_fast<false>(g.x, next_row, g.d_in, 0, a0);
            };
            if (LSTM) {
                mfma_chunk<4>(a0, bp0 + k0 * NC, NC, BH, acc, pf1);
                mfma_chunk<4>(a1, bp0 + (k0 + kBK) * NC, NC, BH, acc, pf0);
            } else {
                mfma_chunk<3>(a0, bp0 + k0 * NC, NC, BH, acc3, pf1);
                mfma_chunk<3>(a1, bp0 + (k0 + kBK) * NC, NC, BH, acc3, pf0);
            }
        }
        // h part: GRU keeps h W_hn apart (accumulator 3) because the reset gate multiplies it
        if (has_h) {
            for (int k0 = 0; k0 < H; k0 += 2 * kBK) {
                auto pf1 = [&] { load_a16_fast<false>(g.h_prev, row, H, k0 + kBK, a1); };
                auto pf0 = [&] {
                    if (k0 + 2 * kBK < H)
                        load_a16_fast<false>(g.h_prev, row, H, k0 + 2 * kBK, a0);
                    else if (next_tile < ntiles)
                        load_a16_fast<false>(g.x, next_row, g.d_in, 0, a0);
                };
                const float *bp = bp0 + (dpad + k0) * NC;
                if (LSTM) {
                    mfma_chunk<4>(a0, bp, NC, BH, acc, pf1);
                    mfma_chunk<4>(a1, bp + kBK * NC, NC, BH, acc, pf0);
                } else {
                    mfma_chunk<2>(a0, bp, NC, BH, acc2, pf1);
                    mfma_chunk<1>(a0, bp + 2 * BH, NC, BH, acc1, NoPrefetch());
                    mfma_chunk<2>(a1, bp + kBK * NC, NC, BH, acc2, pf0);
                    mfma_chunk<1>(a1, bp + kBK * NC + 2 * BH, NC, BH, acc1, NoPrefetch());
                }
            }
        }
        if (j >= H) continue;
        const int64_t rbase = tile * 32 + 4 * kk;
        const bool full = tile * 32 + 32 <= g.n;
        float prev[16];
        const float *pstate = LSTM ? g.c_prev : g.h_prev;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t rr = rbase + 8 * (r / 4) + (r % 4);
            prev[r] = (pstate && (full || rr < g.n)) ? pstate[rr * H + j] : 0.0f;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t rr = rbase + 8 * (r / 4) + (r % 4);
            if (!(full || rr < g.n)) continue;
            const int64_t o = rr * H + j;
            if (LSTM) {
                const float gi = sigmoidf_(acc[0][r] + bi[0] + bh[0]);
                const float gf = sigmoidf_(acc[1][r] + bi[1] + bh[1]);
                const float gg = tanhf(acc[2][r] + bi[2] + bh[2]);
                const float go = sigmoidf_(acc[3][r] + bi[3] + bh[3]);
                const float cn = gf * prev[r] + gi * gg;
                g.c_out[o] = cn;
                g.h_out[o] = go * tanhf(cn);
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
                const float gn = tanhf(acc[2][r] + bi[2] + gr * ghn);
                g.h_out[o] = (1.0f - gz) * gn + gz * prev[r];
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
}

template <bool LSTM, int WN>
bool rnn_fused_resident_launch(const RnnArgs &g, hipStream_t s)
{
    constexpr int KG = LSTM ? 4 : 3;
    constexpr int WM = 8 / WN;
    if (g.d_in % (2 * kBK) != 0 || g.H % (2 * kBK) != 0) return false;
    const size_t lds = size_t(g.d_in + g.H) * KG * 32 * WN * sizeof(float);
    if (lds > kLdsBytes - 1024) return false;
    auto k = rnn_fused_resident_kernel<LSTM, WN>;
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, int(lds)) != hipSuccess)
        return false;
    const int per_cu = resident_blocks(reinterpret_cast<const void *>(k), 512, lds);
    if (per_cu <= 0) return false;
    const int64_t ntiles = (g.n + 31) / 32;
    const unsigned gy = unsigned((g.H + 32 * WN - 1) / (32 * WN));
    dim3 grid(unsigned(std::min<int64_t>((ntiles + WM - 1) / WM, std::max<int64_t>(1, int64_t(kNumCU) * per_cu / gy))), gy);
    k<<<grid, 512, lds, s>>>(g);
    return true;
}

template <bool LSTM>
bool rnn_fused_resident_dispatch(const RnnArgs &g, hipStream_t s)
{
    if (g.H > 64 && rnn_fused_resident_launch<LSTM, 4>(g, s)) return true;
    if (g.H > 32 && rnn_fused_resident_launch<LSTM, 2>(g, s)) return true;
    return rnn_fused_resident_launch<LSTM, 1>(g, s);
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

template <bool HAS_RS>
__global__ void __launch_bounds__(256) gemm_reduce_kernel(ReduceArgs g)
{
    __shared__ float red[3][64 * 65];
    __shared__ float bred[4][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int i = lane & 31, kk = lane >> 5;
    // 1-D grid; consecutive block ids go round the 8 XCDs, so id % 8 picks the XCD.  All slabs of one row chunk
    // are given to the same XCD (and to neighbouring ids), so that chunk's rows are fetched from HBM once and the
    // other slabs find them in that XCD's L2.
    const int slabs_x = (g.K + 63) / 64, slabs = slabs_x * ((g.M + 63) / 64);
#ifdef REINC_REDUCE_SIMPLE_MAP
    const int slab = blockIdx.x % slabs, chunk = blockIdx.x / slabs;
#else
    const int xcd = blockIdx.x % 8, qid = blockIdx.x / 8;
    const int slab = qid % slabs, chunk = (qid / slabs) * 8 + xcd;
#endif
    if (chunk >= g.chunks) return;
    const int f0 = (slab % slabs_x) * 64, c0 = (slab / slabs_x) * 64;
    const int64_t r_begin = int64_t(chunk) * g.rows_per_chunk;
    const int64_t r_end = min(g.n, r_begin + g.rows_per_chunk);
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
    // wave w takes row pairs w, w+4, ... of the chunk, kRU pairs per trip.  Full trips over full 64x64 slabs run
    // without a single branch: every load of the trip is issued before any arithmetic touches a loaded value.
    constexpr int kRU = 8;
    int64_t base = r_begin;
    if (f0 + 64 <= g.K && c0 + 64 <= g.M) {
        const float *ap = g.A + (base + 2 * w + kk) * g.lda + f0 + i;
        const float *gp = g.G + (base + 2 * w + kk) * g.ldg + c0 + i;
        const float *sp = HAS_RS ? g.row_scale + base + 2 * w + kk : nullptr;
        for (; base + 8 * kRU <= r_end; base += 8 * kRU) {
            float a0[kRU], a1[kRU], b0[kRU], b1[kRU], sc[kRU];
#pragma unroll
            for (int u = 0; u < kRU; ++u) {
                a0[u] = ap[int64_t(8 * u) * g.lda];
                a1[u] = ap[int64_t(8 * u) * g.lda + 32];
                b0[u] = gp[int64_t(8 * u) * g.ldg];
                b1[u] = gp[int64_t(8 * u) * g.ldg + 32];
                sc[u] = HAS_RS ? sp[8 * u] : 1.0f;
            }
            ap += int64_t(8 * kRU) * g.lda;
            gp += int64_t(8 * kRU) * g.ldg;
            if (HAS_RS) sp += 8 * kRU;
            __builtin_amdgcn_sched_barrier(0);  // keep every load of the trip ahead of the arithmetic
#pragma unroll
            for (int u = 0; u < kRU; ++u) {
                if (HAS_RS) {
                    a0[u] *= sc[u];
                    a1[u] *= sc[u];
                }
                acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[u], b0[u], acc[0][0], 0, 0, 0);
                acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[u], b1[u], acc[0][1], 0, 0, 0);
                acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[u], b0[u], acc[1][0], 0, 0, 0);
                acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[u], b1[u], acc[1][1], 0, 0, 0);
                bsum[0] += b0[u];
                bsum[1] += b1[u];
            }
        }
    }
    // ragged slabs and the last rows of the chunk: guarded loads
    for (int64_t r0 = base + 2 * w + kk; r0 < r_end + kk; r0 += 8 * kRU) {
        // (the bound keeps both half-waves in step: a half that runs past r_end loads zeros)
        float a0[kRU], a1[kRU], b0[kRU], b1[kRU];
#pragma unroll
        for (int u = 0; u < kRU; ++u) {
            const int64_t r = r0 + 8 * u;
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
    // combine the four waves: waves 1..3 park their slabs in LDS, wave 0 adds them in order
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int fr = 32 * a + 8 * (r / 4) + 4 * kk + (r % 4), cc = 32 * b + i;
                if (w > 0) red[w - 1][fr * 65 + cc] = acc[a][b][r];
            }
    {
        const float s0 = bsum[0] + __shfl_xor(bsum[0], 32), s1 = bsum[1] + __shfl_xor(bsum[1], 32);
        if (kk == 0) {
            bred[w][i] = s0;
            bred[w][32 + i] = s1;
        }
    }
    __syncthreads();
    if (w != 0) return;
    float *out = g.partial + int64_t(chunk) * (g.K + 1) * g.M;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int cc = 32 * b + i;
            float old[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) old[r] = 0.0f;
            if (g.accumulate) {  // all 16 reads of the tile go out together
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int fr = 32 * a + 8 * (r / 4) + 4 * kk + (r % 4);
                    if (f0 + fr < g.K && c0 + cc < g.M) old[r] = out[int64_t(f0 + fr) * g.M + c0 + cc];
                }
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int fr = 32 * a + 8 * (r / 4) + 4 * kk + (r % 4);
                const float v = ((acc[a][b][r] + red[0][fr * 65 + cc]) + red[1][fr * 65 + cc]) + red[2][fr * 65 + cc];
                if (f0 + fr < g.K && c0 + cc < g.M) out[int64_t(f0 + fr) * g.M + c0 + cc] = old[r] + v;
            }
        }
    if (f0 == 0 && c0 + lane < g.M) {
        float *o = out + int64_t(g.K) * g.M + c0 + lane;
        const float v = ((bred[0][lane] + bred[1][lane]) + bred[2][lane]) + bred[3][lane];
        *o = g.accumulate ? *o + v : v;
    }
}

// dst_w[K*M] += sum_c partial[c][0..K*M);  dst_b[M] += sum_c partial[c][K*M ..)
// A block owns 64 consecutive outputs; its 4 waves split the chunks, then add their sums in wave order.
__global__ void __launch_bounds__(256)
reduce_partials_kernel(const float *partial, int chunks, int K, int M, float *dst_w, float *dst_b)
{
    __shared__ float red[4][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int total = (K + 1) * M;
    const int idx = blockIdx.x * 64 + lane;
    float s0 = 0.0f, s1 = 0.0f;
    if (idx < total) {
        int c = w;
        for (; c + 4 < chunks; c += 8) {
            s0 += partial[int64_t(c) * total + idx];
            s1 += partial[int64_t(c + 4) * total + idx];
        }
        if (c < chunks) s0 += partial[int64_t(c) * total + idx];
    }
    red[w][lane] = s0 + s1;
    __syncthreads();
    if (w != 0 || idx >= total) return;
    const float s = ((red[0][lane] + red[1][lane]) + red[2][lane]) + red[3][lane];
    if (idx < K * M)
        dst_w[idx] += s;
    else if (dst_b)
        dst_b[idx - K * M] += s;
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
        const float tc = tanhf(g.c_new[idx]);
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
constexpr int kLossBlocks = 256;

__global__ void __launch_bounds__(256) mse_partial_kernel(const float *h, const float *y, int64_t total, float *partial)
{
    __shared__ float red[256];
    float s = 0.0f;
    for (int64_t i = blockIdx.x * int64_t(256) + threadIdx.x; i < total; i += int64_t(gridDim.x) * 256) {
        const float e = h[i] - y[i];
        s += e * e;
    }
    red[threadIdx.x] = s;
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
    red[threadIdx.x] = int(threadIdx.x) < nparts ? partial[threadIdx.x] : 0.0f;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) loss[0] = red[0] / float(total);
}

__global__ void mse_grad_kernel(const float *h, const float *y, int64_t total, float *dh)
{
    const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
    if (i < total) dh[i] = 2.0f * (h[i] - y[i]) / float(total);
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
    // preferred: weight slab resident in LDS, as wide as fits
    if (M > 64 && gemm_rows_resident_launch<4, 1>(g, a_bf16, s)) return 0;
    if (M > 32 && gemm_rows_resident_launch<REINC_GEMM64_NT, 2 / REINC_GEMM64_NT>(g, a_bf16, s)) return 0;
    if (gemm_rows_resident_launch<1, 1>(g, a_bf16, s)) return 0;
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

void launch_rnn_fused(int lstm, const float *x, int64_t n, int32_t d_in, int32_t H, const float *h_prev,
                      const float *c_prev, const float *W_i, const float *W_h, const float *b_i, const float *b_h,
                      float *h_out, float *c_out, float *saved, hipStream_t s)
{
    if (n <= 0) return;
    RnnArgs g{x, n, d_in, H, h_prev, c_prev, W_i, W_h, b_i, b_h, h_out, c_out, saved};
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

int reduce_chunks(int64_t n, int32_t K, int32_t M)
{
    // about three blocks per compute unit, at least 256 rows each
    const int64_t slabs = int64_t((K + 63) / 64) * ((M + 63) / 64);
    int64_t chunks = std::max<int64_t>(1, (768 + slabs - 1) / slabs);
    chunks = std::min<int64_t>(chunks, (n + 255) / 256);
    return int(std::max<int64_t>(chunks, 1));
}

uint64_t reduce_partial_bytes(int64_t n, int32_t K, int32_t M)
{
    return uint64_t(reduce_chunks(n, K, M)) * uint64_t(K + 1) * M * 4;
}

void launch_gemm_reduce(const float *A, int32_t lda, const float *row_scale, const float *G, int32_t ldg, int64_t n,
                        int32_t K, int32_t M, float *partial, int accumulate, hipStream_t s)
{
    if (n <= 0) return;
    const int chunks = reduce_chunks(n, K, M);
    int64_t rpc = (n + chunks - 1) / chunks;
    rpc = (rpc + 63) & ~int64_t(63);  // whole 64-row trips; no row pair straddles two chunks
    ReduceArgs g{A, lda, row_scale, G, ldg, n, K, M, rpc, partial, chunks, accumulate};
    const int slabs = ((K + 63) / 64) * ((M + 63) / 64);
    const unsigned blocks = unsigned(slabs) * unsigned((chunks + 7) / 8) * 8u;
    if (row_scale)
        gemm_reduce_kernel<true><<<blocks, 256, 0, s>>>(g);
    else
        gemm_reduce_kernel<false><<<blocks, 256, 0, s>>>(g);
}

void launch_reduce_partials(const float *partial, int64_t n, int32_t K, int32_t M, float *dW, float *db, hipStream_t s)
{
    if (n <= 0) return;
    const int total = (K + 1) * M;
    reduce_partials_kernel<<<(total + 63) / 64, 256, 0, s>>>(partial, reduce_chunks(n, K, M), K, M, dW, db);
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
    mse_partial_kernel<<<kLossBlocks, 256, 0, s>>>(h, y, total, partial);
    mse_final_kernel<<<1, 256, 0, s>>>(partial, kLossBlocks, total, loss);
}

void launch_mse_grad(const float *h, const float *y, int64_t total, float *dh, hipStream_t s)
{
    if (total > 0) mse_grad_kernel<<<unsigned((total + 255) / 256), 256, 0, s>>>(h, y, total, dh);
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
