// Statistics of a calibration set for the bias calibration (first two lines of
// Alg. 2): damage weights w[i][t] = |ReLU(W_gate[i,:] x_t) (W_up[i,:] x_t)|^2 ||W_down[:,i]||^2
// and proxy scores s[i][t] = (A B x_t)_i, for T tokens at once.  These are dense
// contractions with reuse (every weight element meets every token), so they run
// on the matrix cores: one LDS-tiled bf16 MFMA kernel, C = A B^T with both
// operands stored K-contiguous, used three times:
//   gate and up against the tokens (two A operands share the B tiles), epilogue -> w;
//   t = X P (against P transposed once), epilogue: t split into three bf16 terms;
//   scores = Q against those terms (A's columns wrap around every r), which is
//   exact to fp32 as in k_scores_mfma.
// Tile: 128 x 128 x 64 per block of four waves, a wave owns 64 x 64 as 4 x 4
// v_mfma_f32_16x16x32_bf16 tiles; global loads of the next K step are in flight
// while the current one is multiplied; LDS rows are padded to nine 16-byte chunks
// so that the sixteen lanes of an operand read hit different banks.
#pragma once

#include "svdp_rows_mfma.h"

namespace svdp {

constexpr int GM_BM = 128, GM_BN = 128, GM_BK = 64;
constexpr int GM_THREADS = 256;
constexpr int GM_STRIDE = GM_BK / 8 + 1;          // 16-byte chunks per LDS row
constexpr int GM_CPT = GM_BM * (GM_BK / 8) / GM_THREADS;     // chunks per thread and tile (4)

enum GemmEpilogue { EPI_DAMAGE = 0, EPI_SPLIT3 = 1, EPI_PLAIN = 2 };

// C[m][n] = sum_k A[m][k % Ka] * B[n][k], k < K.  A1 (and A2 when NA == 2): [M][lda], B: [N][ldb], bf16.
// EPI_DAMAGE: out[m*ldo + n] = (max(c1,0)*c2)^2 * scale[m]          (fp32)
// EPI_SPLIT3: c1 -> three bf16 terms at planes[m*ldo + {0, N, 2N} + n]
// EPI_PLAIN : out[m*ldo + n] = c1
template <int NA, int EPI>
__global__ __launch_bounds__(GM_THREADS, 2) void k_gemm_nt(const bf16 *__restrict__ A1, const bf16 *__restrict__ A2, int lda,
                                                        int Ka, const bf16 *__restrict__ Bm, int ldb, int M, int N, int K,
                                                        const float *__restrict__ scale, float *__restrict__ out,
                                                        uint16_t *__restrict__ planes, int ldo)
{
    __shared__ uint4 sA[NA][GM_BM * GM_STRIDE];
    __shared__ uint4 sB[GM_BN * GM_STRIDE];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lm = lane & 15, lq = lane >> 4;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * GM_BM, n0 = blockIdx.x * GM_BN;

    f32x4_t acc[NA][4][4];
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[a][i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    uint4 ra[NA][GM_CPT], rb[GM_CPT];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int q = 0; q < GM_CPT; ++q) {
            const int id = tid + q * GM_THREADS, row = id >> 3, c = id & 7;
            const int k = k0 + c * 8;
            const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
            const bool kin = k < K;
            const int m = m0 + row, n = n0 + row;
            ra[0][q] = (kin && m < M) ? load_raw(A1 + (size_t)m * lda + (k % Ka)) : zero;
            if (NA == 2) ra[NA - 1][q] = (kin && m < M) ? load_raw(A2 + (size_t)m * lda + (k % Ka)) : zero;
            rb[q] = (kin && n < N) ? load_raw(Bm + (size_t)n * ldb + k) : zero;
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < K; k0 += GM_BK) {
        __syncthreads();                                            // the previous step's reads are done
#pragma unroll
        for (int q = 0; q < GM_CPT; ++q) {
            const int id = tid + q * GM_THREADS, row = id >> 3, c = id & 7;
#pragma unroll
            for (int a = 0; a < NA; ++a) sA[a][row * GM_STRIDE + c] = ra[a][q];
            sB[row * GM_STRIDE + c] = rb[q];
        }
        __syncthreads();
        if (k0 + GM_BK < K) fetch(k0 + GM_BK);
#pragma unroll
        for (int h = 0; h < GM_BK / 32; ++h) {
            uint4 fb[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) fb[j] = sB[(wn * 64 + j * 16 + lm) * GM_STRIDE + h * 4 + lq];
#pragma unroll
            for (int a = 0; a < NA; ++a) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint4 fa = sA[a][(wm * 64 + i * 16 + lm) * GM_STRIDE + h * 4 + lq];
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[a][i][j] = mfma_bf16(fa, fb[j], acc[a][i][j]);
                }
            }
        }
    }

    // the lane holds rows 4*lq .. 4*lq+3 and column lm of each 16 x 16 tile
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int m = m0 + wm * 64 + i * 16 + lq * 4 + e;
            if (m >= M) continue;
            const float sc = EPI == EPI_DAMAGE ? scale[m] : 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = n0 + wn * 64 + j * 16 + lm;
                if (n >= N) continue;
                const float c1 = acc[0][i][j][e];
                if (EPI == EPI_DAMAGE) {
                    const float z = fmaxf(c1, 0.f) * acc[NA - 1][i][j][e];
                    out[(size_t)m * ldo + n] = z * z * sc;
                } else if (EPI == EPI_PLAIN) {
                    out[(size_t)m * ldo + n] = c1;
                } else {
                    const uint32_t hi = bf16_rne_bits(c1);
                    const float r1 = c1 - __uint_as_float(hi << 16);
                    const uint32_t mid = bf16_rne_bits(r1);
                    const float r2 = r1 - __uint_as_float(mid << 16);
                    uint16_t *p = planes + (size_t)m * ldo + n;
                    p[0] = (uint16_t)hi;
                    p[N] = (uint16_t)mid;
                    p[2 * N] = (uint16_t)bf16_rne_bits(r2);
                }
            }
        }
    }
}

// out[i] = sum_j W[i][j]^2 for a bf16 matrix [rows][cols], one wave per row (fixed order).
__global__ __launch_bounds__(256) void k_row_norm2(const bf16 *__restrict__ Wm, int rows, int cols,
                                                   float *__restrict__ out)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    float acc = 0.f;
    for (int v = lane; v < cols / 8; v += 64) {
        float w[8];
        load_vec(Wm + (size_t)row * cols + (size_t)v * 8, w);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc = fmaf(w[e], w[e], acc);
    }
    acc = wave_sum(acc);
    if (lane == 0) out[row] = acc;
}

// dst [cols][rows] = src [rows][cols]^T, 16-bit elements, 32 x 32 tiles through LDS.
__global__ __launch_bounds__(256) void k_transpose16(const uint16_t *__restrict__ src, int rows, int cols,
                                                     uint16_t *__restrict__ dst)
{
    __shared__ uint16_t tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;       // 32 x 8
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    for (int y = ty; y < 32; y += 8)
        if (r0 + y < rows && c0 + tx < cols) tile[y][tx] = src[(size_t)(r0 + y) * cols + c0 + tx];
    __syncthreads();
    for (int y = ty; y < 32; y += 8)
        if (c0 + y < cols && r0 + tx < rows) dst[(size_t)(c0 + y) * rows + r0 + tx] = tile[tx][y];
}

}   // namespace svdp
