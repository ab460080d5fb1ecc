// Offline predictor build with data whitening (Sec. 4.1, Alg. 1), fp64 on the GPU.
//
// Given W_gate [D][d] and calibration tokens X [T][d], Alg. 1 takes a factor S of the
// second-moment matrix (S S^T = X^T X in the row-token convention used here), the SVD of
// W_gate S = U Sigma V^T, and returns A = U_r Sigma_r, B = V_r^T S^-1, the rank-r pair
// minimising ||(W_gate - A B) X^T||_F.  In the library's letters Q = A [D][r], P = B^T [d][r].
//
// Everything that is a dense contraction runs on the matrix cores (k_dgemm_nt, fp64 MFMA),
// including the bulk of the blocked Cholesky factorisation that gives S and of the block
// back-substitution that applies S^-1; the symmetric d x d eigen-decomposition (of (W S)^T (W S), whose
// eigenvectors are V and eigenvalues Sigma^2) is a two-sided BLOCK Jacobi method in which a round
// is ONE pass over the matrix: the blocks of rows and columns that are transformed together are
// neighbours in memory, so a 64 x 64 tile needs only its own elements and the two small orthogonal
// matrices of its row strip and column strip (products on the matrix cores), and the tile is
// written to the places the round-robin pairing wants its blocks in for the next round.
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

// dst[k][j] = src[idx[k]][j] for k < nsel
__global__ __launch_bounds__(256) void k_gather_rows(const double *__restrict__ src, const int32_t *__restrict__ idx,
                                                     int nsel, int cols, double *__restrict__ dst)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (size_t)nsel * cols) return;
    dst[i] = src[(size_t)idx[i / cols] * cols + i % cols];
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

// With Cin the result is Cin - A B^T (Cin [M][ldcin], not the same memory as C).
__global__ __launch_bounds__(256) void k_dgemm_nt(const double *__restrict__ A, int lda, const double *__restrict__ Bm,
                                                  int ldb, double *__restrict__ C, int ldc, int M, int N, int K,
                                                  const double *__restrict__ Cin, int ldcin)
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
                if (m < M && n < N)
                    C[(size_t)m * ldc + n] = Cin != nullptr ? Cin[(size_t)m * ldcin + n] - acc[i][j][v] : acc[i][j][v];
            }
}

// ---------------------------------------------------------------------------
// Blocked Cholesky factorisation C = L L^T (Alg. 1's S), block size 64, left-looking.  Per block column k:
//   T[k:, k] = C[k:, k] - L[k:, :k] L[k, :k]^T         k_dgemm_nt with Cin (T is a scratch matrix)
//   L[k, k]  = chol(T[k, k]), and its inverse           k_chol_diag (one block, in LDS)
//   L[k+1:, k] = T[k+1:, k] L[k, k]^-T                  k_dgemm_nt against the inverse
// The inverses of the diagonal blocks are kept (transposed) for the block back-substitution that applies
// L^-1 to the chosen singular vectors at the end.
// ---------------------------------------------------------------------------
constexpr int CH_B = 64;

// out[0] = largest diagonal element of A [n][n] (one block)
__global__ __launch_bounds__(256) void k_max_diag(const double *__restrict__ A, int n, double *__restrict__ out)
{
    __shared__ double sm[256];
    double m = 0.0;
    for (int i = threadIdx.x; i < n; i += 256) m = fmax(m, A[(size_t)i * n + i]);
    sm[threadIdx.x] = m;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (threadIdx.x < w) sm[threadIdx.x] = fmax(sm[threadIdx.x], sm[threadIdx.x + w]);
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = sm[0];
}

// Lkk (lower, the part above the diagonal zero) = Cholesky factor of the 64 x 64 block at T + toff (row stride n),
// written to L + toff; invL [64][64] = Lkk^-1 and invLt its transpose.  A pivot that is not above tiny * scale[0]
// (the matrix is not positive definite to working precision) sets fail[0] = 1 and is replaced by that bound, so
// that the rest of the run stays finite.
__global__ __launch_bounds__(256) void k_chol_diag(const double *__restrict__ T, double *__restrict__ L, int n,
                                                   size_t toff, const double *__restrict__ scale, double tiny,
                                                   double *__restrict__ invL, double *__restrict__ invLt,
                                                   int *__restrict__ fail)
{
    __shared__ double S[CH_B][CH_B + 1], X[CH_B][CH_B + 1];
    const int tid = threadIdx.x;
    for (int e = tid; e < CH_B * CH_B; e += 256) S[e >> 6][e & 63] = T[toff + (size_t)(e >> 6) * n + (e & 63)];
    const double bound = tiny * scale[0];
    __syncthreads();
    for (int j = 0; j < CH_B; ++j) {
        if (tid == 0) {
            double p = S[j][j];
            if (!(p > bound)) {
                fail[0] = 1;
                p = bound > 0.0 ? bound : 1.0;
            }
            S[j][j] = sqrt(p);
        }
        __syncthreads();
        if (tid > j && tid < CH_B) S[tid][j] /= S[j][j];
        __syncthreads();
        for (int e = tid; e < CH_B * CH_B; e += 256) {
            const int i = e >> 6, c = e & 63;
            if (c > j && i >= c) S[i][c] -= S[i][j] * S[c][j];
        }
        __syncthreads();
    }
    if (tid < CH_B) {                         // column tid of the inverse, by forward substitution
        const int c = tid;
        for (int i = 0; i < CH_B; ++i) {
            double v = 0.0;
            if (i >= c) {
                v = i == c ? 1.0 : 0.0;
                for (int k = c; k < i; ++k) v -= S[i][k] * X[k][c];
                v /= S[i][i];
            }
            X[i][c] = v;
        }
    }
    __syncthreads();
    for (int e = tid; e < CH_B * CH_B; e += 256) {
        const int i = e >> 6, c = e & 63;
        L[toff + (size_t)i * n + c] = c <= i ? S[i][c] : 0.0;
        invL[e] = X[i][c];
        invLt[c * CH_B + i] = X[i][c];
    }
}

// zero above the diagonal blocks of L [n][n] (the blocks on the diagonal are already lower triangular)
__global__ __launch_bounds__(256) void k_zero_upper_blocks(double *__restrict__ L, int n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (size_t)n * n) return;
    const int row = (int)(i / n), col = (int)(i % n);
    if (col / CH_B > row / CH_B) L[i] = 0.0;
}

// ---------------------------------------------------------------------------
// Block Jacobi for a symmetric matrix A [n][n] (n a multiple of 64), eigenvectors accumulated as
// rows of Vt (Vt starts as the identity; at the end A is diagonal up to the tolerance and row i of
// Vt is the eigenvector of A[i][i]).
//
// The matrix is cut into blocks of 32 rows / columns.  One round pairs the blocks (2k, 2k+1) -
// always neighbours, so a pair is the contiguous strip of rows 64k .. 64k+63 - and
//   k_bjacobi_solve  runs a cyclic Jacobi sweep (all 2016 pairs of its 64 indices) over every strip's own
//                    64 x 64 diagonal tile in LDS and stores the accumulated orthogonal U_k;
//   k_bjacobi_apply  forms A <- U^T A U tile by tile (the tile of strip a and strip c needs only
//                    itself, U_a and U_c: two 64 x 64 x 64 products on the fp64 matrix cores) and
//                    Vt <- U^T Vt (one product), and writes every tile straight to the place the
//                    round-robin tournament wants its blocks in for the next round: block 0 stays,
//                    an odd block 2k+1 moves to 2k-1 (block 1 to 2), an even block 2k to 2k+2 (the
//                    last even one to the last place).  After nblocks-1 rounds every pair of blocks
//                    has met once (one sweep); no separate permutation pass exists.
// Against rotating single rows and columns this moves the matrix once per 32 of them.
// ---------------------------------------------------------------------------
constexpr int BJ_B = 32;                 // block size
constexpr int BJ_S = 2 * BJ_B;           // strip / tile size
constexpr int BJ_LD = BJ_S + 1;          // LDS row stride in doubles
// Sweeps over a diagonal tile per round.  More of them bring the tile closer to diagonal but not the matrix:
// on the 4096 x 4096 matrices of the 7B layer the number of outer sweeps stayed 12 to 13 for 1, 2, 4 and 12
// (to convergence) inner sweeps, while the whole factorisation took 0.94, 1.16, 1.46 and 2.29 s.
constexpr int BJ_INNER_SWEEPS = 1;

__device__ __forceinline__ int jacobi_next_place(int i, int n)
{
    if (n <= 2 || i == 0) return i;
    if (i & 1) return i == 1 ? 2 : i - 2;
    return i == n - 2 ? n - 1 : i + 2;
}
// row or column index -> its place after this round (blocks move, offsets inside a block stay)
__device__ __forceinline__ int bjacobi_next_index(int i, int n)
{
    return jacobi_next_place(i / BJ_B, n / BJ_B) * BJ_B + i % BJ_B;
}

// Round-robin tournament over 64 indices: seat 0 holds index 0, seat i >= 1 holds 1 + (i - 1 + step) mod 63, and
// the pairs of a step are the seats (m, 63 - m), m = 0 .. 31.  bj_seat gives a seat's index in step 0, bj_advance
// the index the same seat holds one step later.
__device__ __forceinline__ int bj_seat(int seat) { return seat; }
__device__ __forceinline__ int bj_advance(int idx) { return idx == 0 ? 0 : (idx == BJ_S - 1 ? 1 : idx + 1); }

// (c, s) of the rotation J = [c s; -s c] that (nearly) zeroes the off-diagonal element of [app apq; apq aqq] in
// J^T . J.  The tangent is worked out in single precision with the hardware's reciprocal and square root - its
// error only leaves a residue of about 1e-7 of the element, which the next sweep removes - and (c, s) from it in
// double precision (reciprocal square root refined by two Newton steps), so that c^2 + s^2 = 1 to rounding and
// the accumulated transform stays orthogonal.  This sits on the critical path of every step: it is a few dozen
// instructions, not the several hundred of IEEE double divisions and square roots.
__device__ __forceinline__ void bj_angle(double app, double aqq, double apq, double &c, double &s)
{
    const float num = (float)(aqq - app), den = 2.0f * (float)apq;
    const float tau = num * __builtin_amdgcn_rcpf(den);                      // den == 0: +-inf or NaN
    const float root = __builtin_amdgcn_sqrtf(__builtin_fmaf(tau, tau, 1.0f));
    float t = __builtin_copysignf(__builtin_amdgcn_rcpf(__builtin_fabsf(tau) + root), tau);   // |tau| = inf: 0
    if (!(t == t) || den == 0.0f) t = 0.0f;
    const double td = (double)t, a = __builtin_fma(td, td, 1.0);            // a in [1, 2]
    double y = __builtin_amdgcn_rsq(a);
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const double e = __builtin_fma(-a * y, y, 1.0);                     // 1 - a y^2
        y = __builtin_fma(0.5 * y, e, y);
    }
    c = y;
    s = td * y;
}

// the value the neighbouring lane (lane ^ 1) holds, through the data-parallel path (no LDS round trip)
__device__ __forceinline__ double bj_neighbour(double v)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_update_dpp(0, lo, 0xB1, 0xF, 0xF, false);          // quad_perm [1, 0, 3, 2]
    hi = __builtin_amdgcn_update_dpp(0, hi, 0xB1, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}

// U[k] (64 x 64, row-major), the product of the rotations of BJ_INNER_SWEEPS cyclic sweeps over the k-th diagonal
// tile S of A (the identity if S is already diagonal to rounding).  One block of 1024 threads per strip; S and U live in LDS (dynamic: 2 * 64 * 65 doubles).  A step applies its 32
// disjoint rotations J to the whole tile in ONE pass, S <- J^T S J: a lane owns one column (of the pair lane / 2,
// the first or second index by lane % 2), a wave takes two row pairs, rotates the two rows at its column and
// gets the neighbour column's values from the neighbouring lane for the column rotation.  Every element is read
// and written by exactly one lane, and a wave's 64 lanes always touch 64 different columns of one row, so the
// accesses spread over all LDS banks.  U <- U J is the same column rotation; the angles of the next step are
// computed (32 lanes) while the other waves are in it.
constexpr int BJ_SOLVE_THREADS = 1024;
__global__ __launch_bounds__(BJ_SOLVE_THREADS) void k_bjacobi_solve(const double *__restrict__ A, int n,
                                                                    double *__restrict__ Uall)
{
    extern __shared__ double bj_smem[];
    double *S = bj_smem;                       // [64][65]
    double *U = S + BJ_S * BJ_LD;              // [64][65]
    __shared__ double csv[2][BJ_B][2];
    __shared__ double red[2][BJ_SOLVE_THREADS / 64];
    __shared__ int done;
    constexpr int WAVES = BJ_SOLVE_THREADS / 64, PAIRS = BJ_B / WAVES, ROWS = BJ_S / WAVES;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, k = blockIdx.x;
    const int pb = lane >> 1, second = lane & 1;
    const size_t base = (size_t)(k * BJ_S) * n + (size_t)k * BJ_S;
    for (int e = tid; e < BJ_S * BJ_S; e += BJ_SOLVE_THREADS) {
        const int i = e >> 6, j = e & 63;
        S[i * BJ_LD + j] = A[base + (size_t)i * n + j];
        U[i * BJ_LD + j] = i == j ? 1.0 : 0.0;
    }
    __syncthreads();
    for (int sweep = 0; sweep < BJ_INNER_SWEEPS; ++sweep) {
        // converged when the off-diagonal part is at rounding level of the tile
        double off = 0.0, all = 0.0;
        for (int e = tid; e < BJ_S * BJ_S; e += BJ_SOLVE_THREADS) {
            const int i = e >> 6, j = e & 63;
            const double v = S[i * BJ_LD + j];
            all += v * v;
            if (i != j) off += v * v;
        }
        for (int w = 32; w > 0; w >>= 1) {
            off += __shfl_xor(off, w);
            all += __shfl_xor(all, w);
        }
        if (lane == 0) {
            red[0][wave] = off;
            red[1][wave] = all;
        }
        // this lane's column, this wave's row pairs and (threads 0 .. 31) the pair whose angle the thread works
        // out, all for step 0; advanced step by step below
        int col = second ? bj_seat(BJ_S - 1 - pb) : bj_seat(pb);
        int rp[PAIRS], rq[PAIRS];
#pragma unroll
        for (int e = 0; e < PAIRS; ++e) {
            rp[e] = bj_seat(wave * PAIRS + e);
            rq[e] = bj_seat(BJ_S - 1 - (wave * PAIRS + e));
        }
        int ap = bj_seat(tid & (BJ_B - 1)), aq = bj_seat(BJ_S - 1 - (tid & (BJ_B - 1)));
        __syncthreads();
        if (tid == 0) {
            double o = 0.0, t = 0.0;
            for (int w = 0; w < WAVES; ++w) {
                o += red[0][w];
                t += red[1][w];
            }
            done = (o <= 1e-26 * t) ? 1 : 0;
        }
        if (tid < BJ_B) {
            double c, s;
            bj_angle(S[ap * BJ_LD + ap], S[aq * BJ_LD + aq], S[ap * BJ_LD + aq], c, s);
            csv[0][tid][0] = c;
            csv[0][tid][1] = s;
        }
        __syncthreads();
        if (done) break;
        for (int step = 0; step < BJ_S - 1; ++step) {
            const int cur = step & 1;
            // column rotation of a value v at this lane's column, w the same row's value at the pair's other
            // column:  first column  c v - s w,  second column  c v + s w
            const double cb = csv[cur][pb][0], sb = second ? csv[cur][pb][1] : -csv[cur][pb][1];
            double x[PAIRS], y[PAIRS];
#pragma unroll
            for (int e = 0; e < PAIRS; ++e) {
                x[e] = S[rp[e] * BJ_LD + col];
                y[e] = S[rq[e] * BJ_LD + col];
            }
#pragma unroll
            for (int e = 0; e < PAIRS; ++e) {
                const double ca = csv[cur][wave * PAIRS + e][0], sa = csv[cur][wave * PAIRS + e][1];
                const double xr = ca * x[e] - sa * y[e], yr = sa * x[e] + ca * y[e];
                const double xo = bj_neighbour(xr), yo = bj_neighbour(yr);
                S[rp[e] * BJ_LD + col] = cb * xr + sb * xo;
                S[rq[e] * BJ_LD + col] = cb * yr + sb * yo;
            }
            __syncthreads();
            ap = bj_advance(ap);
            aq = bj_advance(aq);
            if (tid < BJ_B && step + 1 < BJ_S - 1) {
                double c, s;
                bj_angle(S[ap * BJ_LD + ap], S[aq * BJ_LD + aq], S[ap * BJ_LD + aq], c, s);
                csv[cur ^ 1][tid][0] = c;
                csv[cur ^ 1][tid][1] = s;
            }
            double u[ROWS];
#pragma unroll
            for (int e = 0; e < ROWS; ++e) u[e] = U[(wave * ROWS + e) * BJ_LD + col];
#pragma unroll
            for (int e = 0; e < ROWS; ++e) {
                const double uo = bj_neighbour(u[e]);
                U[(wave * ROWS + e) * BJ_LD + col] = cb * u[e] + sb * uo;
            }
            col = bj_advance(col);
#pragma unroll
            for (int e = 0; e < PAIRS; ++e) {
                rp[e] = bj_advance(rp[e]);
                rq[e] = bj_advance(rq[e]);
            }
            __syncthreads();
        }
    }
    for (int e = tid; e < BJ_S * BJ_S; e += BJ_SOLVE_THREADS) {
        const int i = e >> 6, j = e & 63;
        Uall[(size_t)k * BJ_S * BJ_S + e] = U[i * BJ_LD + j];
    }
}

// 64 x 64 x 64 product on the matrix cores, operands in LDS:  C[i][j] = sum_k L(k, i) * R[k][j]  with
// L(k, i) = Lm[k][i] (LT: the left factor is used transposed, U^T T) or Lm[i][k] (X U).  Wave (wm, wn) owns the
// 32 x 32 quadrant; the result register v of a lane is C[16 ti + 4 v + lq][16 tj + lm] of its tile (ti, tj).
template <bool LT>
__device__ __forceinline__ void bj_mma64(const double *Lm, const double *Rm, int wm, int wn, int lm, int lq,
                                         f64x4_t (&acc)[2][2])
{
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = f64x4_t{0.0, 0.0, 0.0, 0.0};
#pragma unroll 4
    for (int kk = 0; kk < BJ_S; kk += 4) {
        double fa[2], fb[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = wm * 32 + i * 16 + lm;
            fa[i] = LT ? Lm[(kk + lq) * BJ_LD + row] : Lm[row * BJ_LD + kk + lq];
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) fb[j] = Rm[(kk + lq) * BJ_LD + wn * 32 + j * 16 + lm];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
}

// TWO_SIDED: out[next(i)][next(j)] = (U_a^T T U_c)[i][j] for the tile T of strip a and strip c (the matrix A);
// otherwise out[next(i)][j] = (U_a^T T)[i][j] (the eigenvector rows Vt).  A block takes `ct` consecutive column
// tiles of one strip: U_a stays in LDS, the next tile's T is on its way from memory into registers while the
// current tile is multiplied, and the lanes' operand values of U_c for the second product are fetched (from L2:
// every block of the column uses them) before the first product starts.  X = U_a^T T takes T's place in LDS, so
// two blocks fit a compute unit and one multiplies while the other loads and stores.
// Dynamic LDS: 2 matrices of 64 x 65 doubles.
template <bool TWO_SIDED>
__global__ __launch_bounds__(256, 2) void k_bjacobi_apply(const double *__restrict__ M, const double *__restrict__ Uall,
                                                          int n, int ct, double *__restrict__ out)
{
    extern __shared__ double bj_smem[];
    double *Ua = bj_smem, *T = Ua + BJ_S * BJ_LD;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lm = lane & 15, lq = lane >> 4, wm = wave >> 1, wn = wave & 1;
    const int a = blockIdx.y, strips = n / BJ_S;
    const int c_begin = blockIdx.x * ct, c_end = min(c_begin + ct, strips);
    constexpr int PER = BJ_S * BJ_S / 256;
    double rt[PER];
    auto fetch = [&](int c) {
#pragma unroll
        for (int e = 0; e < PER; ++e) {
            const int idx = tid + 256 * e, i = idx >> 6, j = idx & 63;
            rt[e] = M[(size_t)(a * BJ_S + i) * n + c * BJ_S + j];
        }
    };
    if (c_begin < c_end) fetch(c_begin);
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int idx = tid + 256 * e;
        Ua[(idx >> 6) * BJ_LD + (idx & 63)] = Uall[(size_t)a * BJ_S * BJ_S + idx];
    }
    for (int c = c_begin; c < c_end; ++c) {
        __syncthreads();            // the previous tile's readers are done with T (holding X)
#pragma unroll
        for (int e = 0; e < PER; ++e) {
            const int idx = tid + 256 * e;
            T[(idx >> 6) * BJ_LD + (idx & 63)] = rt[e];
        }
        __syncthreads();
        if (c + 1 < c_end) fetch(c + 1);
        double ub[BJ_S / 4][2];     // U_c[4 kk + lq][this lane's two columns]
        if (TWO_SIDED) {
#pragma unroll
            for (int kk = 0; kk < BJ_S / 4; ++kk)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    ub[kk][j] = Uall[(size_t)c * BJ_S * BJ_S + (4 * kk + lq) * BJ_S + wn * 32 + j * 16 + lm];
        }
        f64x4_t acc[2][2];
        bj_mma64<true>(Ua, T, wm, wn, lm, lq, acc);
        if (TWO_SIDED) {
            __syncthreads();        // every wave has read T
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        T[(wm * 32 + i * 16 + 4 * v + lq) * BJ_LD + wn * 32 + j * 16 + lm] = acc[i][j][v];
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = f64x4_t{0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int kk = 0; kk < BJ_S / 4; ++kk) {
                double fa[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) fa[i] = T[(wm * 32 + i * 16 + lm) * BJ_LD + 4 * kk + lq];
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(fa[i], ub[kk][j], acc[i][j], 0, 0, 0);
            }
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int row = a * BJ_S + wm * 32 + i * 16 + 4 * v + lq;
                    const int col = c * BJ_S + wn * 32 + j * 16 + lm;
                    out[(size_t)bjacobi_next_index(row, n) * n + (TWO_SIDED ? bjacobi_next_index(col, n) : col)] =
                        acc[i][j][v];
                }
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
