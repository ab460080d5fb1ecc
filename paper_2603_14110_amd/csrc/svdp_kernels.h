// gfx950 kernels of the sparse decode step.  Template parameters:
//   W  : storage element (float or bf16); arithmetic is always fp32
//   NB : compile-time batch capacity (1, 2, 4, 8); the runtime batch B <= NB
// Every floating-point sum below is formed in an order that depends only on
// the launch shape and the index list, never on timing (no fp atomics).
#pragma once

#include "svdp_device.h"

namespace svdp {

constexpr int XP_THREADS = 256;      // k_xP block
constexpr int SC_THREADS = 256;      // k_scores block
constexpr int SC_SLAB = 64;          // neurons per k_scores block = one mask word
constexpr int ROWS_THREADS = 512;    // k_rows block
constexpr int SCAN_THREADS = 1024;   // k_compact_scan block

// ---------------------------------------------------------------------------
// Predictor stage 1: partial t = x P over a slab of rows of P   (Sec. 4.1 eq. 2:
// the inner factor B x of A B x + b, with P = B^T).
// Block g owns rows [g*rows_per_wg, (g+1)*rows_per_wg) of P [d][r] and writes
// tpart[g][b][0..r).  A thread owns one 16-byte column group and every
// nsub-th row of the slab; the nsub row-partials are then added through LDS.
// Dynamic LDS: NB*rows_per_wg + XP_THREADS*VEC*NB floats.
// ---------------------------------------------------------------------------
template <typename W, int NB>
__global__ __launch_bounds__(XP_THREADS) void k_xP(const W *__restrict__ P, const W *__restrict__ x,
                                                   int B, int d, int r, int rows_per_wg,
                                                   float *__restrict__ tpart)
{
    constexpr int VEC = Elem<W>::VEC;
    extern __shared__ float smem[];
    float *xs = smem;                         // [NB][rows_per_wg]
    float *red = smem + NB * rows_per_wg;     // [nsub][NB][r]
    const int tid = threadIdx.x;
    const int cg = r / VEC;                   // column groups, <= XP_THREADS
    const int nsub = XP_THREADS / cg;
    const int j0 = blockIdx.x * rows_per_wg;
    const int j1 = min(d, j0 + rows_per_wg);

    for (int i = tid; i < NB * rows_per_wg; i += XP_THREADS) {
        const int b = i / rows_per_wg, j = j0 + i % rows_per_wg;
        xs[i] = (b < B && j < j1) ? to_f32(x[(size_t)b * d + j]) : 0.f;
    }
    __syncthreads();

    const int cgi = tid % cg, sub = tid / cg;
    float acc[NB][VEC];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[b][e] = 0.f;

    if (sub < nsub) {
        const W *col = P + (size_t)cgi * VEC;
#pragma unroll 4
        for (int j = j0 + sub; j < j1; j += nsub) {
            float w[VEC];
            load_vec(col + (size_t)j * r, w);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const float xv = xs[b * rows_per_wg + (j - j0)];
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[b][e] = fmaf(xv, w[e], acc[b][e]);
            }
        }
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int e = 0; e < VEC; ++e) red[(sub * NB + b) * r + cgi * VEC + e] = acc[b][e];
    }
    __syncthreads();
    for (int c = tid; c < NB * r; c += XP_THREADS) {
        const int b = c / r, k = c % r;
        float s = 0.f;
        for (int q = 0; q < nsub; ++q) s += red[(q * NB + b) * r + k];
        tpart[((size_t)blockIdx.x * NB + b) * r + k] = s;
    }
}

// ---------------------------------------------------------------------------
// Predictor stage 2 + step function: s_i = t . Q[i,:] + b_i for one slab of 64
// neurons, then (optionally) the 64-bit mask word of the slab:
// bit j = OR over tokens of [s > 0]   (eq. 2's H; the union over the batch).
// t is first assembled from the nt stage-1 partials (fixed order) into LDS.
// A group of 2^lpr_log2 lanes owns one row of Q at a time.
// Dynamic LDS: NB*r + NB*64 floats.
// ---------------------------------------------------------------------------
template <typename W, int NB>
__global__ __launch_bounds__(SC_THREADS) void k_scores(const W *__restrict__ Q,
                                                       const float *__restrict__ bias,
                                                       const float *__restrict__ tpart, int nt, int B,
                                                       int D, int r, int lpr_log2,
                                                       float *__restrict__ s_out,
                                                       uint64_t *__restrict__ mask_out)
{
    constexpr int VEC = Elem<W>::VEC;
    extern __shared__ float smem[];
    float *ts = smem;              // [NB][r]
    float *sc = smem + NB * r;     // [NB][64]
    const int tid = threadIdx.x;
    const int i0 = blockIdx.x * SC_SLAB;

    for (int c = tid; c < NB * r; c += SC_THREADS) {
        float s = 0.f;
        for (int g = 0; g < nt; ++g) s += tpart[(size_t)g * NB * r + c];
        ts[c] = s;
    }
    __syncthreads();

    const int lpr = 1 << lpr_log2;
    const int lig = tid & (lpr - 1);
    const int grp = tid >> lpr_log2;
    const int ngrp = SC_THREADS >> lpr_log2;
    const int cg = r / VEC;
    for (int n = grp; n < SC_SLAB; n += ngrp) {
        const W *row = Q + (size_t)(i0 + n) * r;
        float acc[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[b] = 0.f;
        for (int v = lig; v < cg; v += lpr) {
            float w[VEC];
            load_vec(row + v * VEC, w);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const float *tb = ts + b * r + v * VEC;
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[b] = fmaf(tb[e], w[e], acc[b]);
            }
        }
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[b] = group_sum(acc[b], lpr_log2);
        if (lig == 0) {
            const float bi = bias[i0 + n];
#pragma unroll
            for (int b = 0; b < NB; ++b) sc[b * SC_SLAB + n] = acc[b] + bi;
        }
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
        int inc = c;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(inc, o);
            if (lane >= o) inc += t;
        }
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
// SparseDown in one launch; with DENSE the list is 0..D-1, i.e. eq. 1).
// The list of n rows is cut into gridDim.x contiguous chunks; block g handles
// chunk g:
//   phase A: one wave per row: g = W_gate[i].x, u = W_up[i].x (wave reduction),
//            h = ReLU(g)*u to LDS;
//   phase B: every thread owns 16-byte column groups of the output and adds
//            h * W_downT[i][cols] over the chunk in list order -> ypart[g].
// Blocks with an empty chunk write nothing; k_reduce_y knows how many wrote.
// Dynamic LDS: NB*d + NB*max_chunk floats.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int chunk_of(int n, int G) { return (n + G - 1) / G; }

template <typename W, int NB, bool DENSE>
__global__ __launch_bounds__(ROWS_THREADS) void k_rows(const W *__restrict__ Wg, const W *__restrict__ Wu,
                                                       const W *__restrict__ WdT, const W *__restrict__ x,
                                                       int B, int d, int D,
                                                       const int32_t *__restrict__ idx,
                                                       const int32_t *__restrict__ nnz_p, int max_chunk,
                                                       uint32_t flags, float *__restrict__ ypart)
{
    constexpr int VEC = Elem<W>::VEC;
    extern __shared__ float smem[];
    float *xs = smem;              // [NB][d]
    float *hs = smem + NB * d;     // [NB][max_chunk]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int n = DENSE ? D : *nnz_p;
    n = max(0, min(n, D));
    const int chunk = chunk_of(n, gridDim.x);
    const int lo = blockIdx.x * chunk;
    const int hi = min(n, lo + chunk);
    if (lo >= hi) return;
    const bool drelu = (flags & 1u) != 0;
    const bool revalidate = (flags & 2u) != 0;

    for (int i = tid; i < NB * d; i += ROWS_THREADS) {
        const int b = i / d;
        xs[i] = b < B ? to_f32(x[i]) : 0.f;
    }
    __syncthreads();

    const int nvec = d / VEC;
    for (int q = lo + wave; q < hi; q += ROWS_THREADS / 64) {
        const size_t row = DENSE ? (size_t)q : (size_t)idx[q];
        const W *g = Wg + row * d;
        const W *u = Wu + row * d;
        float ag[NB], au[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) ag[b] = au[b] = 0.f;
#pragma unroll 2
        for (int v = lane; v < nvec; v += 64) {
            float wg[VEC], wu[VEC];
            load_vec(g + v * VEC, wg);
            load_vec(u + v * VEC, wu);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const float *xb = xs + b * d + v * VEC;
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    ag[b] = fmaf(wg[e], xb[e], ag[b]);
                    au[b] = fmaf(wu[e], xb[e], au[b]);
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
                hs[b * max_chunk + (q - lo)] = gp * uu;
            }
        }
    }
    __syncthreads();

    for (int v = tid; v < nvec; v += ROWS_THREADS) {
        float acc[NB][VEC];
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[b][e] = 0.f;
#pragma unroll 4
        for (int q = lo; q < hi; ++q) {
            float h[NB];
            bool any = false;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                h[b] = hs[b * max_chunk + (q - lo)];
                any = any || (h[b] != 0.f);
            }
            if (revalidate && !any) continue;
            const size_t row = DENSE ? (size_t)q : (size_t)idx[q];
            float w[VEC];
            load_vec(WdT + row * d + v * VEC, w);
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[b][e] = fmaf(h[b], w[e], acc[b][e]);
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
// y[b][:] = sum over the blocks of k_rows that had work, in block order
// (second stage of the deterministic down-projection reduction, App. C).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_reduce_y(const float *__restrict__ ypart,
                                                  const int32_t *__restrict__ nnz_p, int n_fixed, int D,
                                                  int G, int NB, int B, int d, float *__restrict__ y)
{
    int n = nnz_p != nullptr ? *nnz_p : n_fixed;
    n = max(0, min(n, D));
    const int chunk = chunk_of(n, G);
    const int gact = n > 0 ? (n + chunk - 1) / chunk : 0;
    const int vpt = d / 4;
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= B * vpt) return;
    const int b = t / vpt, v = t % vpt;
    const float4 *src = reinterpret_cast<const float4 *>(ypart) + (size_t)b * vpt + v;
    const size_t stride = (size_t)NB * vpt;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 8
    for (int g = 0; g < gact; ++g) {
        const float4 p = src[(size_t)g * stride];
        s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
    }
    reinterpret_cast<float4 *>(y)[(size_t)b * vpt + v] = s;
}

// ---------------------------------------------------------------------------
// Glue of the stacked benchmark: x_next = (x+y)/sqrt(mean((x+y)^2)+eps) + shift.
// One block; the sum of squares is reduced in a fixed order.
// ---------------------------------------------------------------------------
template <typename W>
__global__ __launch_bounds__(1024) void k_stack_glue(const W *x, const float *__restrict__ y,
                                                     const float *__restrict__ shift, int d, float eps,
                                                     W *x_next)
{
    __shared__ float part[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float ss = 0.f;
    for (int j = tid; j < d; j += 1024) {
        const float v = to_f32(x[j]) + y[j];
        ss = fmaf(v, v, ss);
    }
    ss = wave_sum(ss);
    if (lane == 0) part[wave] = ss;
    __syncthreads();
    float tot = 0.f;
    for (int q = 0; q < 16; ++q) tot += part[q];
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
    __syncthreads();
    for (int j = tid; j < d; j += 1024) {
        const float v = (to_f32(x[j]) + y[j]) * inv + shift[j];
        from_f32(v, &x_next[j]);
    }
}

}  // namespace svdp
