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
};

__global__ void __launch_bounds__(256) gemm_reduce_kernel(ReduceArgs g)
{
    __shared__ float red[3][64 * 65];
    __shared__ float bred[4][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int i = lane & 31, kk = lane >> 5;
    const int f0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
    const int64_t r_begin = int64_t(blockIdx.z) * g.rows_per_chunk;
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
    // wave w takes row pairs w, w+4, ... of the chunk
    for (int64_t r = r_begin + 2 * w + kk; r < r_end + kk; r += 8) {
        // (the loop bound keeps both half-waves in step: the kk = 1 half may see r == r_end and loads zeros)
        const bool live = r < r_end;
        float a0 = 0.0f, a1 = 0.0f, b0 = 0.0f, b1 = 0.0f;
        if (live) {
            const float sc = g.row_scale ? g.row_scale[r] : 1.0f;
            const float *ap = g.A + r * g.lda + f0 + i;
            const float *gp = g.G + r * g.ldg + c0 + i;
            if (fa0) a0 = ap[0] * sc;
            if (fa1) a1 = ap[32] * sc;
            if (cb0) b0 = gp[0];
            if (cb1) b1 = gp[32];
        }
        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
        acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        bsum[0] += b0;
        bsum[1] += b1;
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
    float *out = g.partial + int64_t(blockIdx.z) * (g.K + 1) * g.M;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int fr = 32 * a + 8 * (r / 4) + 4 * kk + (r % 4), cc = 32 * b + i;
                const float v = ((acc[a][b][r] + red[0][fr * 65 + cc]) + red[1][fr * 65 + cc]) + red[2][fr * 65 + cc];
                if (f0 + fr < g.K && c0 + cc < g.M) out[int64_t(f0 + fr) * g.M + c0 + cc] = v;
            }
    if (blockIdx.x == 0 && c0 + lane < g.M)
        out[int64_t(g.K) * g.M + c0 + lane] = ((bred[0][lane] + bred[1][lane]) + bred[2][lane]) + bred[3][lane];
}

// dst_w[K*M] += sum_c partial[c][0..K*M);  dst_b[M] += sum_c partial[c][K*M ..)
__global__ void reduce_partials_kernel(const float *partial, int chunks, int K, int M, float *dst_w, float *dst_b)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    const int total = (K + 1) * M;
    if (idx >= total) return;
    float s = 0.0f;
    for (int c = 0; c < chunks; ++c) s += partial[int64_t(c) * total + idx];
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
    const int64_t slabs = int64_t((K + 63) / 64) * ((M + 63) / 64);
    int64_t chunks = std::max<int64_t>(1, 1024 / slabs);
    chunks = std::min<int64_t>(chunks, (n + 255) / 256);
    return int(std::max<int64_t>(chunks, 1));
}

uint64_t reduce_partial_bytes(int64_t n, int32_t K, int32_t M)
{
    return uint64_t(reduce_chunks(n, K, M)) * uint64_t(K + 1) * M * 4;
}

void launch_gemm_reduce(const float *A, int32_t lda, const float *row_scale, const float *G, int32_t ldg, int64_t n,
                        int32_t K, int32_t M, float *partial, float *dW, float *db, hipStream_t s)
{
    if (n <= 0) return;
    const int chunks = reduce_chunks(n, K, M);
    int64_t rpc = (n + chunks - 1) / chunks;
    rpc = (rpc + 7) & ~int64_t(7);  // whole row-pair groups per wave
    ReduceArgs g{A, lda, row_scale, G, ldg, n, K, M, rpc, partial};
    dim3 grid(unsigned((K + 63) / 64), unsigned((M + 63) / 64), unsigned(chunks));
    gemm_reduce_kernel<<<grid, 256, 0, s>>>(g);
    const int total = (K + 1) * M;
    reduce_partials_kernel<<<(total + 255) / 256, 256, 0, s>>>(partial, chunks, K, M, dW, db);
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

void launch_fill_f32(float *p, int64_t n, float v, hipStream_t s)
{
    if (n > 0) fill_f32_kernel<<<unsigned((n + 255) / 256), 256, 0, s>>>(p, n, v);
}

}  // namespace reinc
