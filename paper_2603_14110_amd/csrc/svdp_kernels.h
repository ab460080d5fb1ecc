// gfx950 kernels of the sparse decode step.  Template parameters:
//   W  : storage element (float or bf16); arithmetic is always fp32
//   NB : compile-time batch capacity (1, 2, 4, 8); the runtime batch B <= NB
// Every floating-point sum below is formed in an order that depends only on
// the launch shape and the index list, never on timing (no fp atomics).
#pragma once

#include "svdp_device.h"

namespace svdp {

constexpr int XP_THREADS = 256;      // k_xP block
constexpr int XP_ROWS = 256;         // rows of P per k_xP block
constexpr int XP_COLS = 32;          // columns of P per k_xP block
constexpr int SC_SLAB = 64;          // neurons per k_scores block = one mask word
constexpr int ROWS_THREADS = 512;    // k_rows block
constexpr int ROWS_WAVES = ROWS_THREADS / 64;
constexpr int ROWS_UB = 4;           // row kernels: rows of W_downT fetched together (the LDS row capacity is padded to this)
constexpr int SCAN_THREADS = 1024;   // k_compact_scan block
constexpr int RED_COLS = 8;          // k_reduce_y: float4 columns per block (one 128-byte line per partial row)
constexpr int RED_SEGS = 64;         // k_reduce_y: segments of the partial list per block

// Sum over j < d of (x[j] + y[j])^2 by a block of 256 threads in a fixed order (a thread takes the
// 16-byte vectors t, t + 256, ... of x in ascending order, then the lanes of a wave, then the four
// waves): the mean square of the stacked benchmark's glue.  Every thread gets the total.
// part: 4 floats of shared memory.  d is a multiple of the vector length.
__device__ __forceinline__ float glue_block_total(float ss, float *part)
{
    const int tid = threadIdx.x;
    ss = wave_sum(ss);
    __syncthreads();
    if ((tid & 63) == 0) part[tid >> 6] = ss;
    __syncthreads();
    return ((part[0] + part[1]) + part[2]) + part[3];
}

template <typename W>
__device__ __forceinline__ float glue_sum_squares(const W *__restrict__ x, const float *__restrict__ y, int d,
                                                  float *part)
{
    constexpr int VEC = Elem<W>::VEC;
    float ss = 0.f;
#pragma unroll 2
    for (int v = threadIdx.x; v < d / VEC; v += 256) {
        float xv[VEC];
        load_vec(x + (size_t)v * VEC, xv);
#pragma unroll
        for (int e4 = 0; e4 < VEC / 4; ++e4) {
            const float4 yv = *reinterpret_cast<const float4 *>(y + (size_t)v * VEC + 4 * e4);
            const float a = xv[4 * e4] + yv.x, b = xv[4 * e4 + 1] + yv.y, c = xv[4 * e4 + 2] + yv.z,
                        dd = xv[4 * e4 + 3] + yv.w;
            ss = fmaf(a, a, ss);
            ss = fmaf(b, b, ss);
            ss = fmaf(c, c, ss);
            ss = fmaf(dd, dd, ss);
        }
    }
    return glue_block_total(ss, part);
}

// ---------------------------------------------------------------------------
// Predictor stage 1: partial t = x P over a tile of P   (Sec. 4.1 eq. 2: the
// inner factor B x of A B x + b, with P = B^T).
// Block (i, j) owns rows [i*XP_ROWS, +XP_ROWS) and columns [j*XP_COLS, +XP_COLS)
// of P [d][r] and writes tpart[i][b][its columns].  A thread owns one 16-byte
// column group and every NSUB-th row of the tile; its loads of P are issued
// before x is staged, and the NSUB row-partials are added through LDS in order.
// Dynamic LDS: NB*XP_ROWS + NSUB*(NB*XP_COLS + 1) + PARTS*NB*XP_COLS floats.
// ---------------------------------------------------------------------------
// With GLUE the token is not given but made here: x = RMSNorm(x_prev + y_prev) + shift rounded to
// the storage type, the stacked benchmark's glue (k_stack_glue forms the mean square with the same
// function, so the two give the same bits).  Every block forms the norm itself from the d sums of x_prev
// and y_prev (a few KB from L2) instead of waiting for one more launch; the blocks of the first
// column tile also write x to x_out for the row kernel.
template <typename W, int NB, bool GLUE>
__global__ __launch_bounds__(XP_THREADS) void k_xP(const W *__restrict__ P, const W *__restrict__ x,
                                                   int B, int d, int r, float *__restrict__ tpart,
                                                   const float *__restrict__ y_prev,
                                                   const float *__restrict__ shift, float eps,
                                                   W *__restrict__ x_out)
{
    constexpr int VEC = Elem<W>::VEC;
    constexpr int CG = XP_COLS / VEC;          // column groups per tile
    constexpr int NSUB = XP_THREADS / CG;      // row phases
    constexpr int RPT = XP_ROWS / NSUB;        // rows per thread
    extern __shared__ float smem[];
    float *xs = smem;                          // [NB][XP_ROWS]
    float *red = smem + NB * XP_ROWS;          // [NSUB][NB*XP_COLS + 1] (odd stride: no bank conflicts)
    const int tid = threadIdx.x;
    const int j0 = blockIdx.x * XP_ROWS;
    const int c0 = blockIdx.y * XP_COLS;
    const int cgi = tid % CG, sub = tid / CG;
    const int col = c0 + cgi * VEC;
    const bool colok = col < r;

    uint4 raw[RPT];
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
        const int j = j0 + sub + k * NSUB;
        if (colok && j < d) raw[k] = load_raw(P + (size_t)j * r + col);
    }
    __shared__ float gpart[4];
    float inv[NB];
    if (GLUE) {
        static_assert(XP_THREADS == 256, "glue_sum_squares is written for 256 threads");
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            inv[b] = 0.f;
            if (b < B) {
                const float tot = glue_sum_squares(x + (size_t)b * d, y_prev + (size_t)b * d, d, gpart);
                inv[b] = 1.0f / sqrtf(tot / (float)d + eps);
            }
        }
    }
    // x of the tile's rows, one 16-byte vector per thread and pass (d is a multiple of VEC)
    for (int i = tid; i < NB * (XP_ROWS / VEC); i += XP_THREADS) {
        const int b = i / (XP_ROWS / VEC), j = j0 + (i % (XP_ROWS / VEC)) * VEC;
        float w[VEC];
        if (b < B && j < d) {
            load_vec(x + (size_t)b * d + j, w);
            if (GLUE) {
                W rounded[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float v = (w[e] + y_prev[(size_t)b * d + j + e]) * inv[b] + shift[j + e];
                    from_f32(v, &rounded[e]);
                    w[e] = to_f32(rounded[e]);
                }
                if (blockIdx.y == 0) {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) x_out[(size_t)b * d + j + e] = rounded[e];
                }
            }
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) w[e] = 0.f;
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) xs[b * XP_ROWS + (j - j0) + e] = w[e];
    }
    __syncthreads();

    float acc[NB][VEC];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[b][e] = 0.f;
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
        const int jj = sub + k * NSUB;
        if (colok && j0 + jj < d) {
            float w[VEC];
            widen(raw[k], w, (const W *)nullptr);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const float xv = xs[b * XP_ROWS + jj];
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[b][e] = fmaf(xv, w[e], acc[b][e]);
            }
        }
    }
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int e = 0; e < VEC; ++e) red[sub * (NB * XP_COLS + 1) + b * XP_COLS + cgi * VEC + e] = acc[b][e];
    __syncthreads();
    // two-level sum of the NSUB row phases (fixed order): the NB*XP_COLS outputs of the
    // tile are shared out over the block, PARTS threads per output
    constexpr int OUTS = NB * XP_COLS;
    constexpr int PARTS = XP_THREADS / OUTS >= 1 ? XP_THREADS / OUTS : 1;
    constexpr int PER = NSUB / PARTS;
    float *red2 = red + NSUB * (OUTS + 1);                   // [PARTS][OUTS]
    for (int o = tid % OUTS, part = tid / OUTS; part < PARTS; part += XP_THREADS) {
        float s = 0.f;
#pragma unroll 8
        for (int q = 0; q < PER; ++q) s += red[(part * PER + q) * (OUTS + 1) + o];
        red2[part * OUTS + o] = s;
    }
    __syncthreads();
    for (int o = tid; o < OUTS; o += XP_THREADS) {
        const int b = o / XP_COLS, k = o % XP_COLS;
        if (c0 + k < r) {
            float t = 0.f;
#pragma unroll
            for (int q = 0; q < PARTS; ++q) t += red2[q * OUTS + o];
            tpart[((size_t)blockIdx.x * NB + b) * r + c0 + k] = t;
        }
    }
}

// ---------------------------------------------------------------------------
// Sum of the nt stage-1 partials into one t (fixed order).  Used for batches of
// four or more tokens, where re-adding the partials in every score block would
// cost more than this extra launch.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_tsum(const float *__restrict__ tpart, int nt, int count,
                                              float *__restrict__ t)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= count) return;
    float s = 0.f;
#pragma unroll 8
    for (int g = 0; g < nt; ++g) s += tpart[(size_t)g * count + c];
    t[c] = s;
}

// ---------------------------------------------------------------------------
// Predictor stage 2 + step function: s_i = t . Q[i,:] + b_i for one slab of 64
// neurons, then (optionally) the 64-bit mask word of the slab:
// bit j = OR over tokens of [s > 0]   (eq. 2's H; the union over the batch).
// A group of LPR = 2^LPR_LOG2 lanes owns every NGRP-th row of the slab; a lane
// owns the column groups lig, lig+LPR, ... of its rows.  The rows' first column
// groups are requested first; then t is assembled from the nt stage-1 partials
// (threads split the partial list, all loads in flight, fixed combination
// order through LDS), so the memory latencies overlap.
// SC_THREADS is 512 for one or two tokens (short critical path) and 256 for larger
// batches (fewer wavefronts repeating the per-wave overhead).
// Dynamic LDS: NB*r + NB*64 + max(SC_THREADS*4, NB*r) floats.
// ---------------------------------------------------------------------------
template <typename W, int NB, int LPR_LOG2, int SC_THREADS>
__global__ __launch_bounds__(SC_THREADS) void k_scores(const W *__restrict__ Q,
                                                       const float *__restrict__ bias,
                                                       const float *__restrict__ tpart, int nt, int B,
                                                       int D, int r, float *__restrict__ s_out,
                                                       uint64_t *__restrict__ mask_out)
{
    constexpr int VEC = Elem<W>::VEC;
    constexpr int LPR = 1 << LPR_LOG2;              // lanes per row: 8, 16, 32 or 64
    constexpr int NGRP = SC_THREADS / LPR;          // lane groups per block
    constexpr int RPG = (SC_SLAB + NGRP - 1) / NGRP;   // rows per lane group (groups beyond the slab idle)
    extern __shared__ float smem[];
    float *ts = smem;                  // [NB][r]
    float *sc = ts + NB * r;           // [NB][64]
    float *tsp = sc + NB * SC_SLAB;    // [npg][NB*r] partial sums of t
    const int tid = threadIdx.x;
    const int i0 = blockIdx.x * SC_SLAB;
    const int lig = tid & (LPR - 1);
    const int grp = tid >> LPR_LOG2;
    const int cg = r / VEC;
    const float my_bias = tid < SC_SLAB ? bias[i0 + tid] : 0.f;     // added after the row sums

    // first column group of each of this group's rows
    uint4 raw[RPG];
    const bool has_rows = NGRP <= SC_SLAB || grp < SC_SLAB;
    const W *qrow = Q + (size_t)(i0 + (has_rows ? grp : 0)) * r + (lig < cg ? lig : 0) * VEC;
#pragma unroll
    for (int k = 0; k < RPG; ++k) raw[k] = load_raw(qrow + (size_t)k * NGRP * r);

    {   // t = sum of the stage-1 partials
        const int ncq = NB * r / 4;                        // float4 columns of t
        const int npg = max(1, SC_THREADS / ncq);          // threads per column
        const float4 *tp4 = reinterpret_cast<const float4 *>(tpart);
        float4 *tsp4 = reinterpret_cast<float4 *>(tsp);
        for (int it = tid; it < ncq * npg; it += SC_THREADS) {
            const int cq = it % ncq, pg = it / ncq;
            float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 8
            for (int g = pg; g < nt; g += npg) {
                const float4 p = tp4[(size_t)g * ncq + cq];
                s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
            }
            tsp4[pg * ncq + cq] = s;
        }
        __syncthreads();
        float4 *ts4 = reinterpret_cast<float4 *>(ts);
        for (int c = tid; c < ncq; c += SC_THREADS) {
            float4 s = tsp4[c];
            for (int pg = 1; pg < npg; ++pg) {
                const float4 p = tsp4[pg * ncq + c];
                s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
            }
            ts4[c] = s;
        }
        __syncthreads();
    }

    float acc[RPG][NB];
#pragma unroll
    for (int k = 0; k < RPG; ++k)
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[k][b] = 0.f;
    if (lig < cg) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            float tv[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) tv[e] = ts[b * r + lig * VEC + e];
#pragma unroll
            for (int k = 0; k < RPG; ++k) {
                float w[VEC];
                widen(raw[k], w, (const W *)nullptr);
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[k][b] = fmaf(tv[e], w[e], acc[k][b]);
            }
        }
    }
    for (int v = lig + LPR; v < cg && has_rows; v += LPR) {          // only when r/VEC > 64
        for (int k = 0; k < RPG; ++k) {
            float w[VEC];
            load_vec(Q + (size_t)(i0 + grp + k * NGRP) * r + v * VEC, w);
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[k][b] = fmaf(ts[b * r + v * VEC + e], w[e], acc[k][b]);
        }
    }
#pragma unroll
    for (int k = 0; k < RPG; ++k)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const float t = group_sum<LPR_LOG2>(acc[k][b]);
            if (lig == 0 && has_rows) sc[b * SC_SLAB + grp + k * NGRP] = t;
        }
    __syncthreads();
    if (tid < SC_SLAB) {
#pragma unroll
        for (int b = 0; b < NB; ++b) sc[b * SC_SLAB + tid] += my_bias;
    }
    __syncthreads();

    if (s_out != nullptr) {
        for (int c = tid; c < NB * SC_SLAB; c += SC_THREADS) {
            const int b = c / SC_SLAB, n = c % SC_SLAB;
            if (b < B) s_out[(size_t)b * D + i0 + n] = sc[c];
        }
    }
    if (mask_out != nullptr && tid < 64) {
        bool on = false;
        for (int b = 0; b < B; ++b) on = on || (sc[b * SC_SLAB + tid] > 0.f);
        const uint64_t m = __ballot(on);
        if (tid == 0) mask_out[blockIdx.x] = m;
    }
}

// ---------------------------------------------------------------------------
// Mask words from materialised scores: one wave per word, bit j of word k is
// neuron 64k + j, set iff s[t][64k+j] > 0 for some token t.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_mask_from_scores(const float *__restrict__ s, int B, int D,
                                                          uint64_t *__restrict__ mask)
{
    const int lane = threadIdx.x & 63;
    const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (k >= D / 64) return;
    bool on = false;
    for (int b = 0; b < B; ++b) on = on || (s[(size_t)b * D + (size_t)k * 64 + lane] > 0.f);
    const uint64_t m = __ballot(on);
    if (lane == 0) mask[k] = m;
}

// ---------------------------------------------------------------------------
// Mask words -> ascending index list and its length (Alg. 4's nonzero).
// One block: popcount per word, block-wide exclusive scan (wave scan +
// 16 wave totals), then one wave per word writes its set bits at
// offset[word] + (number of set bits below the lane).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(SCAN_THREADS) void k_compact_scan(const uint64_t *__restrict__ mask,
                                                               int nwords, int32_t *__restrict__ idx,
                                                               int32_t *__restrict__ nnz)
{
    __shared__ int wsum[SCAN_THREADS / 64];
    __shared__ int offs[SCAN_THREADS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int running = 0;
    for (int base = 0; base < nwords; base += SCAN_THREADS) {
        const int k = base + tid;
        const uint64_t w = k < nwords ? mask[k] : 0ull;
        const int c = __popcll(w);
        const int inc = wave_inclusive_scan(c);
        if (lane == 63) wsum[wave] = inc;
        __syncthreads();
        int wbase = 0, tot = 0;
        for (int q = 0; q < SCAN_THREADS / 64; ++q) {
            const int s = wsum[q];
            if (q < wave) wbase += s;
            tot += s;
        }
        offs[tid] = running + wbase + inc - c;
        __syncthreads();
        const int nw_here = min(SCAN_THREADS, nwords - base);
        for (int kk = wave; kk < nw_here; kk += SCAN_THREADS / 64) {
            const uint64_t ww = mask[base + kk];
            if ((ww >> lane) & 1ull) {
                const int below = __popcll(ww & ((1ull << lane) - 1ull));
                idx[offs[kk] + below] = (base + kk) * 64 + lane;
            }
        }
        running += tot;
        __syncthreads();
    }
    if (tid == 0) *nnz = running;
}

// ---------------------------------------------------------------------------
// Gate, up and down over a list of rows (Alg. 3's SparseGate / SparseUpAndMul /
// SparseDown in one launch).  Where the list comes from:
//   ROWS_DENSE : all D rows (eq. 1, the dense baseline)
//   ROWS_LIST  : idx_in[0 .. *nnz_in)           (svdp_sparse_ffn)
//   ROWS_MASK  : the set bits of mask[0 .. D/64) (svdp_ffn_step): every block
//                scans the popcounts of the mask words itself (Alg. 4's
//                nonzero, without a separate launch) and extracts its own
//                part of the ascending list; when idx_out / nnz_out are given
//                each block also writes its part of the list there.
// The list of n rows is cut into gridDim.x contiguous chunks; block g handles
// chunk g:
//   phase A: one wave per row: g = W_gate[i].x, u = W_up[i].x (wave reduction),
//            h = ReLU(g)*u to LDS;
//   phase B: every thread owns 16-byte column groups of the output and adds
//            h * W_downT[i][cols] over the chunk in list order -> ypart[g].
//            The first rows of W_downT are requested before phase A starts.
// Blocks with an empty chunk write nothing; block 0 records n for k_reduce_y.
// max_chunk (the LDS row capacity) is a multiple of ROWS_UB.
// Dynamic LDS: NB*d storage elements (x as stored), NB*max_chunk floats, max_chunk ints.
// ---------------------------------------------------------------------------
enum RowsMode { ROWS_DENSE = 0, ROWS_LIST = 1, ROWS_MASK = 2 };

// Rows per block: the list of n rows is cut into contiguous chunks of
// max(min_chunk, ceil(n / G)) rows, so that a short list occupies fewer blocks and leaves
// fewer partial y's to write and sum.  (Spreading a list of ~1000 rows of the 7B shape over every
// compute unit is 0.3 us faster in the row kernel than four rows per block and 1.3 us faster than
// eight, measured; four costs the step nothing, because the sum of the partials gains what the
// row kernel loses, and halves the partial-y traffic of short lists.)
__device__ __forceinline__ int chunk_of(int n, int G, int min_chunk) { return max(min_chunk, (n + G - 1) / G); }
// Blocks that get rows (= partial y's written).
__device__ __forceinline__ int active_blocks(int n, int chunk) { return n > 0 ? (n + chunk - 1) / chunk : 0; }

// Length n of the row list.  ROWS_MASK: every wave scans the popcounts of all mask words
// by itself (lane l owns the wpl consecutive words starting at l*wpl), so no block-wide
// step is needed; lane_first is the list position of the lane's first set bit.  The
// lane's first ROWS_WREG words stay in registers (held[]) for rows_list_from_mask.
constexpr int ROWS_WREG = 4;        // covers D <= 16384
template <int MODE>
__device__ __forceinline__ int rows_list_length(int D, const uint64_t *__restrict__ mask,
                                                const int32_t *__restrict__ nnz_in, int lane, int &lane_first,
                                                int &wpl, uint64_t (&held)[ROWS_WREG])
{
    lane_first = 0;
    wpl = 0;
    if (MODE == ROWS_DENSE) return D;
    if (MODE == ROWS_LIST) return max(0, min(*nnz_in, D));
    const int nwords = D / 64;
    wpl = (nwords + 63) / 64;
    int c = 0;
#pragma unroll
    for (int j = 0; j < ROWS_WREG; ++j) {
        const int k = lane * wpl + j;
        held[j] = (j < wpl && k < nwords) ? mask[k] : 0ull;
        c += __popcll(held[j]);
    }
    for (int j = ROWS_WREG; j < wpl; ++j) {
        const int k = lane * wpl + j;
        if (k < nwords) c += __popcll(mask[k]);
    }
    const int inc = wave_inclusive_scan(c);
    lane_first = inc - c;
    return __builtin_amdgcn_readlane(inc, 63);
}

// Entries [lo, hi) of the ascending list of set mask bits -> lidx[0 .. hi-lo), by one wave.
// Lane l knows where its words start in the list (lane_first).  Words that overlap
// [lo, hi) are handed to the whole wave one at a time: lane j then looks at bit j, whose
// list position is the word's start plus the number of set bits below it.
__device__ __forceinline__ void rows_list_word(uint64_t w, int j, int wpl, int lane, int &p, int lo, int hi, int *lidx)
{
    const int pc = __popcll(w);
    const bool overlaps = pc > 0 && p < hi && p + pc > lo;
    uint64_t todo = __ballot(overlaps);
    while (todo != 0ull) {
        const int src = __ffsll((unsigned long long)todo) - 1;
        todo &= todo - 1ull;
        const uint32_t wlo = __builtin_amdgcn_readlane((uint32_t)w, src);
        const uint32_t whi = __builtin_amdgcn_readlane((uint32_t)(w >> 32), src);
        const int pk = __builtin_amdgcn_readlane(p, src);
        const uint64_t wk = ((uint64_t)whi << 32) | wlo;
        if ((wk >> lane) & 1ull) {
            const int pos = pk + __popcll(wk & ((1ull << lane) - 1ull));
            if (pos >= lo && pos < hi) lidx[pos - lo] = (src * wpl + j) * 64 + lane;
        }
    }
    p += pc;
}
__device__ __forceinline__ void rows_list_from_mask(int D, const uint64_t *__restrict__ mask, int lane,
                                                    int lane_first, int wpl, const uint64_t (&held)[ROWS_WREG], int lo,
                                                    int hi, int *lidx)
{
    const int nwords = D / 64;
    int p = lane_first;
#pragma unroll
    for (int j = 0; j < ROWS_WREG; ++j)
        if (j < wpl) rows_list_word(held[j], j, wpl, lane, p, lo, hi, lidx);
    for (int j = ROWS_WREG; j < wpl; ++j) {
        const int k = lane * wpl + j;
        rows_list_word(k < nwords ? mask[k] : 0ull, j, wpl, lane, p, lo, hi, lidx);
    }
}

// This block's part of the row list into lidx[0 .. cnt): from the caller's list (entries outside
// [0, D) become -1 and are skipped by every row kernel: they contribute nothing), from the mask
// words (wave 0), or the block's own range of all rows.  Ends with a block barrier.
template <int MODE>
__device__ __forceinline__ void rows_block_list(int D, const uint64_t *__restrict__ mask,
                                                const int32_t *__restrict__ idx_in, int lane_first, int wpl,
                                                const uint64_t (&held)[ROWS_WREG], int lo, int hi, int *lidx)
{
    const int tid = threadIdx.x, cnt = hi - lo;
    if (MODE == ROWS_LIST) {
        for (int q = tid; q < cnt; q += blockDim.x) {
            const int i = idx_in[lo + q];
            lidx[q] = (unsigned)i < (unsigned)D ? i : -1;
        }
    } else if (MODE == ROWS_MASK) {
        if (tid < 64) rows_list_from_mask(D, mask, tid, lane_first, wpl, held, lo, hi, lidx);
    } else {
        for (int q = tid; q < cnt; q += blockDim.x) lidx[q] = lo + q;
    }
    __syncthreads();
}

template <typename W, int NB, int MODE>
__global__ __launch_bounds__(ROWS_THREADS) __attribute__((amdgpu_waves_per_eu(4))) void k_rows(
    const W *__restrict__ Wg, const W *__restrict__ Wu, const W *__restrict__ WdT, const W *__restrict__ x, int B,
    int d, int D, const uint64_t *__restrict__ mask, const int32_t *__restrict__ idx_in,
    const int32_t *__restrict__ nnz_in, int32_t *__restrict__ idx_out, int32_t *__restrict__ nnz_out,
    int32_t *__restrict__ n_used, int max_chunk, int min_chunk, uint32_t flags, float *__restrict__ ypart)
{
    constexpr int VEC = Elem<W>::VEC;
    constexpr int UA = NB <= 2 ? 8 : 4;     // 16-byte loads in flight per matrix in phase A
    constexpr int UB = ROWS_UB;             // rows of W_downT per group in phase B
    extern __shared__ uint4 smem16[];
    const int nvec = d / VEC;
    uint4 *xraw = smem16;                                        // [NB][nvec] x in storage form
    float *hs = reinterpret_cast<float *>(xraw + NB * nvec);     // [NB][max_chunk]
    int *lidx = reinterpret_cast<int *>(hs + NB * max_chunk);    // [max_chunk]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int G = gridDim.x;

    // ---- request x (as stored, no conversion; rows of a batch beyond B are zero).  The first
    // vector of every token stays in registers until the list is known, so that the request
    // for the mask words below is in flight together with it ----
    uint4 xfirst[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
        xfirst[b] = (b < B && tid < nvec) ? load_raw(x + (size_t)b * d + (size_t)tid * VEC) : make_uint4(0u, 0u, 0u, 0u);

    // ---- the list: n, this block's chunk [lo, hi) ----
    int lane_first, wpl;
    uint64_t held[ROWS_WREG];
    const int n = rows_list_length<MODE>(D, mask, nnz_in, lane, lane_first, wpl, held);
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (tid < nvec) xraw[b * nvec + tid] = xfirst[b];
        for (int v = tid + ROWS_THREADS; v < nvec; v += ROWS_THREADS)
            xraw[b * nvec + v] = b < B ? load_raw(x + (size_t)b * d + (size_t)v * VEC) : make_uint4(0u, 0u, 0u, 0u);
    }
    const int chunk = chunk_of(n, G, min_chunk);
    const int lo = min(n, (int)blockIdx.x * chunk);
    const int hi = min(n, lo + chunk);
    const int cnt = hi - lo;
    if (blockIdx.x == 0 && tid == 0) {
        if (MODE != ROWS_DENSE) *n_used = n;
        if (MODE == ROWS_MASK && nnz_out != nullptr) *nnz_out = n;
    }
    if (cnt <= 0) return;

    // h of the positions past the chunk's end (phase B works in whole groups of UB rows)
    const int ngroups = (cnt + UB - 1) / UB;
    for (int i = cnt + tid; i < ngroups * UB; i += ROWS_THREADS)
#pragma unroll
        for (int b = 0; b < NB; ++b) hs[b * max_chunk + i] = 0.f;
    rows_block_list<MODE>(D, mask, idx_in, lane_first, wpl, held, lo, hi, lidx);
    if (MODE == ROWS_MASK && idx_out != nullptr)
        for (int q = tid; q < cnt; q += ROWS_THREADS) idx_out[lo + q] = lidx[q];

    const bool drelu = (flags & 1u) != 0;
    // row q of the chunk, or -1 (past the end; a rejected entry of the caller's list)
    auto row_of = [&](int q) -> int { return q < cnt ? (MODE == ROWS_DENSE ? lo + q : lidx[q]) : -1; };
    auto down_piece = [&](int q, const W *colp) -> uint4 {      // the same branch for every thread of the block
        const int row = row_of(q);
        uint4 piece = make_uint4(0u, 0u, 0u, 0u);
        if (row >= 0) piece = load_raw(colp + (size_t)row * d);
        return piece;
    };

    // ---- request the first group of W_downT rows for this thread's first column group ----
    uint4 cur[UB];
    if (tid < nvec) {
#pragma unroll
        for (int k = 0; k < UB; ++k) cur[k] = down_piece(k, WdT + (size_t)tid * VEC);
    }

    // ---- phase A: one wave per row; the row's 16-byte vectors are fetched UA at a time per
    // matrix and lane (the whole row at once when d <= 64*UA*VEC) ----
    for (int q = wave; q < cnt; q += ROWS_WAVES) {
        const int row = row_of(q);
        float ag[NB], au[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) ag[b] = au[b] = 0.f;
        if (row >= 0) {
            const W *g = Wg + (size_t)row * d;
            const W *u = Wu + (size_t)row * d;
            // whole batches of UA vectors per matrix and lane, then one batch with a ragged end
            int vb = 0;
            for (; vb + 64 * UA <= nvec; vb += 64 * UA) {
                uint4 rg[UA], ru[UA];
#pragma unroll
                for (int k = 0; k < UA; ++k) {
                    rg[k] = load_raw(g + (size_t)(vb + k * 64 + lane) * VEC);
                    ru[k] = load_raw(u + (size_t)(vb + k * 64 + lane) * VEC);
                }
#pragma unroll
                for (int k = 0; k < UA; ++k) {
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        const uint4 xv = xraw[b * nvec + vb + k * 64 + lane];
                        ag[b] = dot_raw(rg[k], xv, ag[b], (const W *)nullptr);
                        au[b] = dot_raw(ru[k], xv, au[b], (const W *)nullptr);
                    }
                }
            }
            if (vb < nvec) {
                uint4 rg[UA], ru[UA];
#pragma unroll
                for (int k = 0; k < UA; ++k) {
                    const int v = vb + k * 64 + lane;
                    rg[k] = ru[k] = make_uint4(0u, 0u, 0u, 0u);
                    if (v < nvec) {
                        rg[k] = load_raw(g + (size_t)v * VEC);
                        ru[k] = load_raw(u + (size_t)v * VEC);
                    }
                }
#pragma unroll
                for (int k = 0; k < UA; ++k) {
                    const int v = min(vb + k * 64 + lane, nvec - 1);      // a zero weight vector meets any x
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        const uint4 xv = xraw[b * nvec + v];
                        ag[b] = dot_raw(rg[k], xv, ag[b], (const W *)nullptr);
                        au[b] = dot_raw(ru[k], xv, au[b], (const W *)nullptr);
                    }
                }
            }
        }
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const float gs = wave_sum(ag[b]);
            const float us = wave_sum(au[b]);
            if (lane == 0) {
                const float gp = fmaxf(gs, 0.f);
                const float uu = drelu ? fmaxf(us, 0.f) : us;
                hs[b * max_chunk + q] = row >= 0 ? gp * uu : 0.f;
            }
        }
    }
    __syncthreads();

    // ---- phase B: every thread owns 16-byte column groups of the output ----
    for (int v = tid; v < nvec; v += ROWS_THREADS) {
        float acc[NB][VEC];
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[b][e] = 0.f;
        const W *colp = WdT + (size_t)v * VEC;
        if (v != tid) {
#pragma unroll
            for (int k = 0; k < UB; ++k) cur[k] = down_piece(k, colp);
        }
        for (int gq = 0; gq < ngroups; ++gq) {
            uint4 nxt[UB];
            if (gq + 1 < ngroups) {
#pragma unroll
                for (int k = 0; k < UB; ++k) nxt[k] = down_piece((gq + 1) * UB + k, colp);
            }
#pragma unroll
            for (int k = 0; k < UB; ++k) {
                float w[VEC];
                widen(cur[k], w, (const W *)nullptr);
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const float h = hs[b * max_chunk + gq * UB + k];
#pragma unroll
                    for (int e = 0; e < VEC; ++e) acc[b][e] = fmaf(h, w[e], acc[b][e]);
                }
            }
#pragma unroll
            for (int k = 0; k < UB; ++k) cur[k] = nxt[k];
        }
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            float4 *out = reinterpret_cast<float4 *>(ypart + ((size_t)blockIdx.x * NB + b) * d + (size_t)v * VEC);
#pragma unroll
            for (int e4 = 0; e4 < VEC / 4; ++e4)
                out[e4] = make_float4(acc[b][4 * e4], acc[b][4 * e4 + 1], acc[b][4 * e4 + 2], acc[b][4 * e4 + 3]);
        }
    }
}

// ---------------------------------------------------------------------------
// y[b][:] = sum over the blocks of the row kernel that had rows (second stage of
// the deterministic down-projection reduction, App. C).
// A block owns RED_COLS float4 columns (one 128-byte line) of one token; the list
// of partials is cut into RED_SEGS contiguous segments summed by different
// threads (all loads in flight at once); the eight segments of a wave are then
// combined with lane shifts, the eight waves through LDS.  The order depends
// only on the number of partials.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float seg8_sum(float v)
{
    v += dpp_move<0x128>(v);        // row_ror:8  -> lanes l and l^8
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}

__global__ __launch_bounds__(RED_COLS *RED_SEGS) void k_reduce_y(const float *__restrict__ ypart,
                                                                 const int32_t *__restrict__ n_ptr, int n_fixed,
                                                                 int D, int G, int min_chunk, int NB, int B, int d,
                                                                 float *__restrict__ y)
{
    static_assert(RED_COLS == 8, "a wave holds 8 columns x 8 segments");
    __shared__ float4 wred[RED_COLS * RED_SEGS / 64][RED_COLS];
    int n = n_ptr != nullptr ? *n_ptr : n_fixed;
    n = max(0, min(n, D));
    const int gact = active_blocks(n, chunk_of(n, G, min_chunk));
    const int vpt = d / 4;
    const int bpt = (vpt + RED_COLS - 1) / RED_COLS;
    const int b = blockIdx.x / bpt;
    const int c = threadIdx.x % RED_COLS, seg = threadIdx.x / RED_COLS;
    const int v = (blockIdx.x % bpt) * RED_COLS + c;
    const int per = (gact + RED_SEGS - 1) / RED_SEGS;
    const int g0 = seg * per, g1 = min(gact, g0 + per);
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (v < vpt) {
        const float4 *src = reinterpret_cast<const float4 *>(ypart) + (size_t)b * vpt + v;
        const size_t stride = (size_t)NB * vpt;
#pragma unroll 4
        for (int g = g0; g < g1; ++g) {
            const float4 p = src[(size_t)g * stride];
            s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
        }
    }
    s.x = seg8_sum(s.x); s.y = seg8_sum(s.y); s.z = seg8_sum(s.z); s.w = seg8_sum(s.w);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane < RED_COLS) wred[wave][lane] = s;
    __syncthreads();
    if (threadIdx.x < RED_COLS && v < vpt) {
        float4 t = wred[0][c];
#pragma unroll
        for (int q = 1; q < RED_COLS * RED_SEGS / 64; ++q) {
            const float4 p = wred[q][c];
            t.x += p.x; t.y += p.y; t.z += p.z; t.w += p.w;
        }
        reinterpret_cast<float4 *>(y)[(size_t)b * vpt + v] = t;
    }
}

// ---------------------------------------------------------------------------
// Glue of the stacked benchmark: x_next = (x+y)/sqrt(mean((x+y)^2)+eps) + shift.
// One block; the sum of squares is reduced in a fixed order.
// ---------------------------------------------------------------------------
template <typename W>
__global__ __launch_bounds__(256) void k_stack_glue(const W *x, const float *__restrict__ y,
                                                    const float *__restrict__ shift, int d, float eps, W *x_next)
{
    constexpr int VEC = Elem<W>::VEC;
    constexpr int KEEP = 4;                            // vectors of x + y a thread keeps in registers
    __shared__ float part[4];
    const int tid = threadIdx.x, nvec = d / VEC;
    // one trip to memory for x, y and the shift of the thread's first KEEP vectors; the sum of squares
    // in the order of glue_sum_squares (the thread's vectors ascending, their elements ascending)
    float v[KEEP][VEC], sh[KEEP][VEC];
#pragma unroll
    for (int k = 0; k < KEEP; ++k) {
        const int vi = tid + k * 256;
        if (vi < nvec) {
            load_vec(x + (size_t)vi * VEC, v[k]);
#pragma unroll
            for (int e4 = 0; e4 < VEC / 4; ++e4) {
                const float4 yv = *reinterpret_cast<const float4 *>(y + (size_t)vi * VEC + 4 * e4);
                const float4 sv = *reinterpret_cast<const float4 *>(shift + (size_t)vi * VEC + 4 * e4);
                v[k][4 * e4] += yv.x; v[k][4 * e4 + 1] += yv.y; v[k][4 * e4 + 2] += yv.z; v[k][4 * e4 + 3] += yv.w;
                sh[k][4 * e4] = sv.x; sh[k][4 * e4 + 1] = sv.y; sh[k][4 * e4 + 2] = sv.z; sh[k][4 * e4 + 3] = sv.w;
            }
        }
    }
    float ss = 0.f;
#pragma unroll
    for (int k = 0; k < KEEP; ++k)
        if (tid + k * 256 < nvec) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) ss = fmaf(v[k][e], v[k][e], ss);
        }
    for (int vi = tid + KEEP * 256; vi < nvec; vi += 256) {
        float xv[VEC];
        load_vec(x + (size_t)vi * VEC, xv);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const float a = xv[e] + y[(size_t)vi * VEC + e];
            ss = fmaf(a, a, ss);
        }
    }
    const float tot = glue_block_total(ss, part);      // its barriers: every read of x above is done (x_next may alias x)
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
    auto emit = [&](int vi, const float (&vv)[VEC], const float (&ss4)[VEC]) {
        W outv[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) from_f32(vv[e] * inv + ss4[e], &outv[e]);
        *reinterpret_cast<uint4 *>(x_next + (size_t)vi * VEC) = *reinterpret_cast<const uint4 *>(outv);
    };
#pragma unroll
    for (int k = 0; k < KEEP; ++k)
        if (tid + k * 256 < nvec) emit(tid + k * 256, v[k], sh[k]);
    for (int vi = tid + KEEP * 256; vi < nvec; vi += 256) {   // a thread rewrites only the vector it reads here
        float xv[VEC], sv[VEC];
        load_vec(x + (size_t)vi * VEC, xv);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            xv[e] += y[(size_t)vi * VEC + e];
            sv[e] = shift[(size_t)vi * VEC + e];
        }
        emit(vi, xv, sv);
    }
}

}  // namespace svdp
