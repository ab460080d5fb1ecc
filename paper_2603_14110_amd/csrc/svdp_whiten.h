// Offline predictor build with data whitening (Sec. 4.1, Alg. 1), fp64 on the GPU.
//
// Given W_gate [D][d] and calibration tokens X [T][d], Alg. 1 takes a factor S of the
// second-moment matrix (S S^T = X^T X in the row-token convention used here), the SVD of
// W_gate S = U Sigma V^T, and returns A = U_r Sigma_r, B = V_r^T S^-1, the rank-r pair
// minimising ||(W_gate - A B) X^T||_F.  In the library's letters Q = A [D][r], P = B^T [d][r].
//
// Everything that is a dense contraction runs on the matrix cores (k_dgemm_nt, fp64 MFMA);
// the two symmetric d x d eigen-decompositions (of X^T X, and of (W S)^T (W S), whose
// eigenvectors are V and eigenvalues Sigma^2) are a cyclic two-sided Jacobi method in which a
// rotation step is ONE pass over the matrix: rows and columns that are rotated together are
// neighbours in memory, so a 64 x 64 tile needs only its own elements and the angles of its 32
// row pairs and 32 column pairs, and the tile is written to the places the round-robin pairing
// wants its rows and columns in for the next step.
#pragma once

#include "svdp_device.h"

namespace svdp {

typedef double f64x4_t __attribute__((ext_vector_type(4)));

// ---- element-wise helpers ----

// dst[i] = (double) src[i]
template <typename W>
__global__ __launch_bounds__(256) void k_to_f64(const W *__restrict__ src, size_t n, double *__restrict__ dst)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = (double)to_f32(src[i]);
}

// dst [cols][rows] (fp64) = src [rows][cols]^T, 32 x 32 tiles through LDS.
template <typename T>
__device__ __forceinline__ double as_f64(T v) { return (double)to_f32(v); }
__device__ __forceinline__ double as_f64(double v) { return v; }

template <typename T>
__global__ __launch_bounds__(256) void k_transpose_to_f64(const T *__restrict__ src, int rows, int cols,
                                                          double *__restrict__ dst)
{
    __shared__ double tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;       // 32 x 8
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    for (int y = ty; y < 32; y += 8)
        if (r0 + y < rows && c0 + tx < cols) tile[y][tx] = as_f64(src[(size_t)(r0 + y) * cols + c0 + tx]);
    __syncthreads();
    for (int y = ty; y < 32; y += 8)
        if (c0 + y < cols && r0 + tx < rows) dst[(size_t)(c0 + y) * rows + r0 + tx] = tile[tx][y];
}

// dst[i][j] = src[i][j] * f(scale[i]) for a [rows][cols] fp64 matrix; POW = 1: sqrt, -1: 1/sqrt
template <int POW>
__global__ __launch_bounds__(256) void k_scale_rows(const double *__restrict__ src, const double *__restrict__ scale,
                                                    int rows, int cols, double *__restrict__ dst)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (size_t)rows * cols) return;
    const double s = sqrt(scale[i / cols]);
    dst[i] = POW > 0 ? src[i] * s : src[i] / s;
}

// dst[k][j] = src[idx[k]][j] * (colscale ? 1/sqrt(colscale[j]) : 1) for k < nsel
__global__ __launch_bounds__(256) void k_gather_rows(const double *__restrict__ src, const int32_t *__restrict__ idx,
                                                     int nsel, int cols, const double *__restrict__ colscale,
                                                     double *__restrict__ dst)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (size_t)nsel * cols) return;
    const int k = (int)(i / cols), j = (int)(i % cols);
    double v = src[(size_t)idx[k] * cols + j];
    if (colscale != nullptr) v /= sqrt(colscale[j]);
    dst[i] = v;
}

__global__ __launch_bounds__(256) void k_f64_to_f32(const double *__restrict__ src, size_t n, float *__restrict__ dst)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = (float)src[i];
}

// ---------------------------------------------------------------------------
// C [M][ldc] = A [M][lda] * B [N][ldb]^T over K (both operands K-contiguous), fp64, on
// v_mfma_f64_16x16x4_f64.  Block tile 64 x 64 x 16, four waves of 32 x 32 (2 x 2 MFMA tiles);
// the next K step's global loads are in flight while the current one is multiplied.
// Operand lanes: A[row = lane%16][k = lane/16], B[k = lane/16][col = lane%16]; the result
// register v of a lane is C[row = 4*v + lane/16][col = lane%16].
// ---------------------------------------------------------------------------
constexpr int DG_BM = 64, DG_BN = 64, DG_BK = 16;
constexpr int DG_LD = DG_BK + 1;            // LDS row stride in doubles (odd: spreads the banks)

__global__ __launch_bounds__(256) void k_dgemm_nt(const double *__restrict__ A, int lda, const double *__restrict__ Bm,
                                                  int ldb, double *__restrict__ C, int ldc, int M, int N, int K)
{
    __shared__ double sA[DG_BM * DG_LD];
    __shared__ double sB[DG_BN * DG_LD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lm = lane & 15, lq = lane >> 4;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * DG_BM, n0 = blockIdx.x * DG_BN;
    // a thread moves four consecutive k of one row of each operand per K step
    const int lrow = tid >> 2, lk = (tid & 3) * 4;

    f64x4_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = f64x4_t{0.0, 0.0, 0.0, 0.0};

    double ra[4], rb[4];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int k = k0 + lk + e;
            ra[e] = (m0 + lrow < M && k < K) ? A[(size_t)(m0 + lrow) * lda + k] : 0.0;
            rb[e] = (n0 + lrow < N && k < K) ? Bm[(size_t)(n0 + lrow) * ldb + k] : 0.0;
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < K; k0 += DG_BK) {
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            sA[lrow * DG_LD + lk + e] = ra[e];
            sB[lrow * DG_LD + lk + e] = rb[e];
        }
        __syncthreads();
        if (k0 + DG_BK < K) fetch(k0 + DG_BK);
#pragma unroll
        for (int kk = 0; kk < DG_BK; kk += 4) {
            double fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) fa[i] = sA[(wm * 32 + i * 16 + lm) * DG_LD + kk + lq];
#pragma unroll
            for (int j = 0; j < 2; ++j) fb[j] = sB[(wn * 32 + j * 16 + lm) * DG_LD + kk + lq];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int m = m0 + wm * 32 + i * 16 + 4 * v + lq;
                const int n = n0 + wn * 32 + j * 16 + lm;
                if (m < M && n < N) C[(size_t)m * ldc + n] = acc[i][j][v];
            }
}

// ---------------------------------------------------------------------------
// Cyclic Jacobi for a symmetric matrix A [n][n] (n a multiple of 64), eigenvectors accumulated
// as rows of Vt (Vt starts as the identity; at the end A is diagonal up to the tolerance and row
// i of Vt is the eigenvector of A[i][i]).
//
// One step rotates the n/2 disjoint pairs (2k, 2k+1): A <- J^T A J, Vt <- J^T Vt with
// J = diag of [[c, s], [-s, c]] blocks, the angle of a pair chosen to annihilate A[2k][2k+1].
// The round-robin tournament then needs new neighbours: index 0 stays, an odd index 2k+1 moves to
// 2k-1 (index 1 to 2), an even index 2k to 2k+2 (the last even one to n-1).  The kernels write
// their results straight to those places, so that after n-1 steps every pair has met once (one
// sweep) and no separate permutation pass exists.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int jacobi_next_place(int i, int n)
{
    if (i == 0) return 0;
    if (i & 1) return i == 1 ? 2 : i - 2;
    return i == n - 2 ? n - 1 : i + 2;
}

// (c, s) of every pair from the 2 x 2 diagonal blocks (the symmetric Schur decomposition)
__global__ __launch_bounds__(256) void k_jacobi_angles(const double *__restrict__ A, int n, double *__restrict__ cs)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= n / 2) return;
    const int p = 2 * k, q = p + 1;
    const double app = A[(size_t)p * n + p], aqq = A[(size_t)q * n + q], apq = A[(size_t)p * n + q];
    double c = 1.0, s = 0.0;
    if (apq != 0.0) {
        const double tau = (aqq - app) / (2.0 * apq);
        const double t = tau >= 0.0 ? 1.0 / (tau + sqrt(1.0 + tau * tau)) : -1.0 / (-tau + sqrt(1.0 + tau * tau));
        c = 1.0 / sqrt(1.0 + t * t);
        s = t * c;
    }
    cs[2 * k] = c;
    cs[2 * k + 1] = s;
}

// out[place(i)][place(j)] = (J^T A J)[i][j] for one 64 x 64 tile
__global__ __launch_bounds__(256) void k_jacobi_rotate(const double *__restrict__ A, const double *__restrict__ cs, int n,
                                                       double *__restrict__ out)
{
    __shared__ double tile[64][65];
    __shared__ double rc[32], rs[32], cc[32], csn[32];
    const int tid = threadIdx.x;
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    if (tid < 32) {
        rc[tid] = cs[r0 + 2 * tid];
        rs[tid] = cs[r0 + 2 * tid + 1];
    } else if (tid < 64) {
        cc[tid - 32] = cs[c0 + 2 * (tid - 32)];
        csn[tid - 32] = cs[c0 + 2 * (tid - 32) + 1];
    }
    for (int e = tid; e < 64 * 64; e += 256) {
        const int i = e >> 6, j = e & 63;
        tile[i][j] = A[(size_t)(r0 + i) * n + c0 + j];
    }
    __syncthreads();
    // rows: pair k = tid / 8, eight columns each
    {
        const int k = tid >> 3, j0 = (tid & 7) * 8;
        const double c = rc[k], s = rs[k];
#pragma unroll
        for (int j = j0; j < j0 + 8; ++j) {
            const double x = tile[2 * k][j], y = tile[2 * k + 1][j];
            tile[2 * k][j] = c * x - s * y;
            tile[2 * k + 1][j] = s * x + c * y;
        }
    }
    __syncthreads();
    // columns: row i = tid / 4, eight column pairs each; straight to the next step's places
    {
        const int i = tid >> 2, k0 = (tid & 3) * 8;
        const size_t orow = (size_t)jacobi_next_place(r0 + i, n) * n;
#pragma unroll
        for (int k = k0; k < k0 + 8; ++k) {
            const double c = cc[k], s = csn[k];
            const double x = tile[i][2 * k], y = tile[i][2 * k + 1];
            out[orow + jacobi_next_place(c0 + 2 * k, n)] = c * x - s * y;
            out[orow + jacobi_next_place(c0 + 2 * k + 1, n)] = s * x + c * y;
        }
    }
}

// out[place(i)][:] = (J^T Vt)[i][:]: one block per row pair
__global__ __launch_bounds__(256) void k_jacobi_rows(const double *__restrict__ Vt, const double *__restrict__ cs, int n,
                                                     double *__restrict__ out)
{
    const int k = blockIdx.x;
    const double c = cs[2 * k], s = cs[2 * k + 1];
    const double *x = Vt + (size_t)(2 * k) * n, *y = x + n;
    double *ox = out + (size_t)jacobi_next_place(2 * k, n) * n, *oy = out + (size_t)jacobi_next_place(2 * k + 1, n) * n;
    for (int j = threadIdx.x; j < n; j += 256) {
        const double a = x[j], b = y[j];
        ox[j] = c * a - s * b;
        oy[j] = s * a + c * b;
    }
}

__global__ __launch_bounds__(256) void k_identity(double *__restrict__ Vt, int n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < (size_t)n * n) Vt[i] = (i / n == i % n) ? 1.0 : 0.0;
}

// sums[0] = sum of squares of the off-diagonal elements, sums[1] = of all elements (one block
// per row, partial sums in a fixed order; the row sums are added by k_jacobi_norms_finish)
__global__ __launch_bounds__(256) void k_jacobi_norms(const double *__restrict__ A, int n, double *__restrict__ rowsums)
{
    __shared__ double so[256], sa[256];
    const int i = blockIdx.x;
    double off = 0.0, all = 0.0;
    for (int j = threadIdx.x; j < n; j += 256) {
        const double v = A[(size_t)i * n + j];
        all += v * v;
        if (j != i) off += v * v;
    }
    so[threadIdx.x] = off;
    sa[threadIdx.x] = all;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (threadIdx.x < w) {
            so[threadIdx.x] += so[threadIdx.x + w];
            sa[threadIdx.x] += sa[threadIdx.x + w];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        rowsums[2 * i] = so[0];
        rowsums[2 * i + 1] = sa[0];
    }
}
__global__ __launch_bounds__(256) void k_jacobi_norms_finish(const double *__restrict__ rowsums, int n,
                                                             const double *__restrict__ A, double *__restrict__ sums,
                                                             double *__restrict__ diag)
{
    __shared__ double so[256], sa[256];
    double off = 0.0, all = 0.0;
    for (int i = threadIdx.x; i < n; i += 256) {
        off += rowsums[2 * i];
        all += rowsums[2 * i + 1];
        diag[i] = A[(size_t)i * n + i];
    }
    so[threadIdx.x] = off;
    sa[threadIdx.x] = all;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (threadIdx.x < w) {
            so[threadIdx.x] += so[threadIdx.x + w];
            sa[threadIdx.x] += sa[threadIdx.x + w];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        sums[0] = so[0];
        sums[1] = sa[0];
    }
}

}   // namespace svdp
