// The whole decode step of Alg. 3 in ONE persistent launch: one block of 1024
// threads per compute unit walks through the four stages
//   1  partial t = x P per tile of P            (Sec. 4.1, eq. 2, inner factor)
//   2  scores of a slab of 64 neurons -> one mask word (eq. 2's step function)
//   3  list of the block's active rows, gate/up/down over them -> partial y
//   4  fixed-order sum of the partial y's for a slice of the columns
// Stages hand their (small) results to every other block through global memory:
// producers write them through to memory (agent-scope stores), wait for the
// writes to complete and bump a counter; consumers poll the counters and read
// the results with agent-scope loads.  No floating-point atomics: every sum is
// formed in a fixed order, so the output is bit-reproducible (App. C).
//
// All blocks must be resident at once (grid <= number of CUs, checked by the
// host); every wait is bounded, and a wait that runs out sets an error flag
// instead of hanging.  The last block to leave zeroes the counters, so a control
// block that starts zeroed is zero again after every launch.
#pragma once

#include "svdp_kernels.h"

namespace svdp {

constexpr int FUSED_THREADS = 1024;
constexpr int FUSED_WAVES = FUSED_THREADS / 64;
__device__ __forceinline__ float group_sum_rt(float v, int log2_lanes)
{
    if (log2_lanes >= 1) v += dpp_move<0xB1>(v);
    if (log2_lanes >= 2) v += dpp_move<0x4E>(v);
    if (log2_lanes >= 3) v += dpp_move<0x141>(v);
    if (log2_lanes >= 4) v += dpp_move<0x140>(v);
    if (log2_lanes >= 5) v += __shfl_xor(v, 16);
    if (log2_lanes >= 6) v += __shfl_xor(v, 32);
    return v;
}

// element j of token b of the staged x, as fp32
__device__ __forceinline__ float staged_x(const uint4 *xraw, int b, int d, int j, const float *)
{
    return reinterpret_cast<const float *>(xraw)[b * d + j];
}
__device__ __forceinline__ float staged_x(const uint4 *xraw, int b, int d, int j, const bf16 *)
{
    return __uint_as_float(((uint32_t) reinterpret_cast<const uint16_t *>(xraw)[b * d + j]) << 16);
}

// half a 16-byte vector: the column group one thread owns in the down projection
__device__ __forceinline__ void widen_half(const uint2 &q, float (&v)[2], const float *)
{
    v[0] = __uint_as_float(q.x); v[1] = __uint_as_float(q.y);
}
__device__ __forceinline__ void widen_half(const uint2 &q, float (&v)[4], const bf16 *)
{
    v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
    v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
}

template <typename W, int NB>
__global__ __launch_bounds__(FUSED_THREADS) void k_step_fused(
    const W *__restrict__ P, const W *__restrict__ Q, const float *__restrict__ bias, const W *__restrict__ Wg,
    const W *__restrict__ Wu, const W *__restrict__ WdT, const W *__restrict__ x, int B, int d, int D, int r,
    int lpr_log2, uint32_t flags, float *tpart, uint64_t *maskbuf, float *ypart, int max_chunk, float *__restrict__ y,
    uint64_t *__restrict__ mask_out, int32_t *__restrict__ idx_out, int32_t *__restrict__ nnz_out, uint32_t *ctrl,
    int spin_limit)
{
    constexpr int VEC = Elem<W>::VEC;
    constexpr int HV = VEC / 2;                 // elements per thread and row in the down projection
    constexpr int UA = NB <= 2 ? 8 : 4;
    constexpr int UB = ROWS_UB;
    constexpr int XCG = XP_COLS / VEC;          // stage 1: column groups per tile
    constexpr int XNSUB = 256 / XCG;            // stage 1: row phases (256 threads work on a tile)
    constexpr int XRPT = XP_ROWS / XNSUB;       // stage 1: rows per thread
    constexpr int MAXRPG = 4;                   // stage 2: rows per lane group (64 rows / 16 groups of 64 lanes)
    extern __shared__ uint4 smem16[];
    const int nvec = d / VEC;
    uint4 *xraw = smem16;                                   // [NB][nvec]  x as stored, whole kernel
    float *scratch = reinterpret_cast<float *>(xraw + NB * nvec);   // reused by every stage
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bid = blockIdx.x, G = gridDim.x;
    const int nt = (d + XP_ROWS - 1) / XP_ROWS, ncs = (r + XP_COLS - 1) / XP_COLS;
    const int ntiles = nt * ncs;
    const int nslabs = D / SC_SLAB;
    const int cg = r / VEC;
    SVDP_STAMP(0, 0);

    // ================= loads that depend on nothing: Q rows of the first slab, P tile, x =================
    const int lpr = 1 << lpr_log2;
    const int lig = tid & (lpr - 1), grp = tid >> lpr_log2;
    const int ngrp = FUSED_THREADS >> lpr_log2;                   // 16 .. 128
    const int rpg = (SC_SLAB + ngrp - 1) / ngrp;                  // 1 .. 4
    const bool has_rows = grp < SC_SLAB;
    uint4 qraw[MAXRPG];
    float my_bias = 0.f;
    if (bid < nslabs) {
        const W *qrow = Q + (size_t)(bid * SC_SLAB + (has_rows ? grp : 0)) * r + (lig < cg ? lig : 0) * VEC;
#pragma unroll
        for (int k = 0; k < MAXRPG; ++k)
            if (k < rpg) qraw[k] = load_raw(qrow + (size_t)k * ngrp * r);
        if (tid < SC_SLAB) my_bias = bias[bid * SC_SLAB + tid];
    }
    const int xcgi = tid % XCG, xsub = (tid & 255) / XCG;
    uint4 praw[XRPT];
    if (bid < ntiles && tid < 256) {
        const int j0 = (bid / ncs) * XP_ROWS, col = (bid % ncs) * XP_COLS + xcgi * VEC;
#pragma unroll
        for (int k = 0; k < XRPT; ++k) {
            const int j = j0 + xsub + k * XNSUB;
            if (col < r && j < d) praw[k] = load_raw(P + (size_t)j * r + col);
        }
    }
#pragma unroll
    for (int b = 0; b < NB; ++b)
        for (int v = tid; v < nvec; v += FUSED_THREADS)
            xraw[b * nvec + v] = b < B ? load_raw(x + (size_t)b * d + (size_t)v * VEC) : make_uint4(0u, 0u, 0u, 0u);
    __syncthreads();

    // ================= stage 1: tiles of t = x P =================
    for (int ti = bid; ti < ntiles; ti += G) {
        const int j0 = (ti / ncs) * XP_ROWS, c0 = (ti % ncs) * XP_COLS;
        const int col = c0 + xcgi * VEC;
        float *red = scratch;                                  // [XNSUB][NB][XP_COLS]
        if (tid < 256) {
            if (ti != bid) {
#pragma unroll
                for (int k = 0; k < XRPT; ++k) {
                    const int j = j0 + xsub + k * XNSUB;
                    if (col < r && j < d) praw[k] = load_raw(P + (size_t)j * r + col);
                }
            }
            float acc[NB][VEC];
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[b][e] = 0.f;
#pragma unroll
            for (int k = 0; k < XRPT; ++k) {
                const int j = j0 + xsub + k * XNSUB;
                if (col < r && j < d) {
                    float w[VEC];
                    widen(praw[k], w, (const W *)nullptr);
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        const float xv = staged_x(xraw, b, d, j, (const W *)nullptr);
#pragma unroll
                        for (int e = 0; e < VEC; ++e) acc[b][e] = fmaf(xv, w[e], acc[b][e]);
                    }
                }
            }
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int e = 0; e < VEC; ++e) red[(xsub * NB + b) * XP_COLS + xcgi * VEC + e] = acc[b][e];
        }
        __syncthreads();
        // two-level sum of the XNSUB row phases (fixed order)
        constexpr int PARTS = 256 / XP_COLS, PER = XNSUB / PARTS;
        const int k = tid % XP_COLS, part = (tid & 255) / XP_COLS;
        for (int b = 0; b < NB; ++b) {
            float s = 0.f;
            if (tid < 256) {
#pragma unroll
                for (int q = 0; q < PER; ++q) s += red[((part * PER + q) * NB + b) * XP_COLS + k];
            }
            __syncthreads();
            if (tid < 256) red[(part * NB + b) * XP_COLS + k] = s;
            __syncthreads();
            if (tid < 256 && part == 0 && c0 + k < r) {
                float t = 0.f;
#pragma unroll
                for (int q = 0; q < PARTS; ++q) t += red[(q * NB + b) * XP_COLS + k];
                store_wt(tpart + ((size_t)(ti / ncs) * NB + b) * r + c0 + k, t);
            }
            __syncthreads();
        }
        wait_stores_done();
        __syncthreads();
        if (tid == 0) signal(ctrl, CTRL_T, ti);
    }

    SVDP_STAMP(0, 1);
    // ================= stage 2: scores of a slab -> mask word =================
    if (bid < nslabs) {
        wait_stage(ctrl, CTRL_T, ntiles, spin_limit);
        SVDP_STAMP(0, 2);
        float *ts = scratch;                         // [NB][r]
        float *sc = ts + NB * r;                     // [NB][64]
        float *tsp = sc + NB * SC_SLAB;              // [npg][NB*r]
        {
            const int ncq = NB * r / 4;
            const int npg = max(1, FUSED_THREADS / ncq);
            float4 *tsp4 = reinterpret_cast<float4 *>(tsp);
            for (int it = tid; it < ncq * npg; it += FUSED_THREADS) {
                const int cq = it % ncq, pg = it / ncq;
                float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
                for (int g = pg; g < nt; g += npg) {
                    const float4 p = load_wt4(tpart + ((size_t)g * ncq + cq) * 4);
                    s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
                }
                tsp4[pg * ncq + cq] = s;
            }
            __syncthreads();
            float4 *ts4 = reinterpret_cast<float4 *>(ts);
            for (int c = tid; c < ncq; c += FUSED_THREADS) {
                float4 s = tsp4[c];
                for (int pg = 1; pg < npg; ++pg) {
                    const float4 p = tsp4[pg * ncq + c];
                    s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
                }
                ts4[c] = s;
            }
            __syncthreads();
        }
        for (int sl = bid; sl < nslabs; sl += G) {
            const int i0 = sl * SC_SLAB;
            if (sl != bid) {
                const W *qrow = Q + (size_t)(i0 + (has_rows ? grp : 0)) * r + (lig < cg ? lig : 0) * VEC;
#pragma unroll
                for (int k = 0; k < MAXRPG; ++k)
                    if (k < rpg) qraw[k] = load_raw(qrow + (size_t)k * ngrp * r);
                my_bias = tid < SC_SLAB ? bias[i0 + tid] : 0.f;
            }
#pragma unroll
            for (int k = 0; k < MAXRPG; ++k) {
                if (k < rpg) {
                    float acc[NB];
#pragma unroll
                    for (int b = 0; b < NB; ++b) acc[b] = 0.f;
                    if (lig < cg && has_rows) {
                        float w[VEC];
                        widen(qraw[k], w, (const W *)nullptr);
#pragma unroll
                        for (int b = 0; b < NB; ++b)
#pragma unroll
                            for (int e = 0; e < VEC; ++e) acc[b] = fmaf(ts[b * r + lig * VEC + e], w[e], acc[b]);
                    }
                    if (has_rows) {
                        const W *row = Q + (size_t)(i0 + grp + k * ngrp) * r;
                        for (int v = lig + lpr; v < cg; v += lpr) {      // only when r/VEC > 64
                            float w[VEC];
                            load_vec(row + v * VEC, w);
#pragma unroll
                            for (int b = 0; b < NB; ++b)
#pragma unroll
                                for (int e = 0; e < VEC; ++e) acc[b] = fmaf(ts[b * r + v * VEC + e], w[e], acc[b]);
                        }
                    }
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        const float t = group_sum_rt(acc[b], lpr_log2);
                        if (lig == 0 && has_rows) sc[b * SC_SLAB + grp + k * ngrp] = t;
                    }
                }
            }
            __syncthreads();
            if (tid < 64) {
                bool on = false;
                for (int b = 0; b < B; ++b) on = on || (sc[b * SC_SLAB + tid] + my_bias > 0.f);
                const uint64_t m = __ballot(on);
                if (tid == 0) {
                    __hip_atomic_store(maskbuf + sl, m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (mask_out != nullptr) mask_out[sl] = m;
                    wait_stores_done();
                    signal(ctrl, CTRL_M, sl);
                }
            }
            __syncthreads();
        }
    }

    SVDP_STAMP(0, 3);
    // ================= stage 3: this block's rows =================
    wait_stage(ctrl, CTRL_M, nslabs, spin_limit);
    SVDP_STAMP(0, 4);
    const int nwords = D / 64;
    uint64_t *mw = reinterpret_cast<uint64_t *>(scratch);                   // [nwords]
    float *hs = reinterpret_cast<float *>(mw + ((nwords + 1) & ~1));        // [NB][max_chunk]
    int *lidx = reinterpret_cast<int *>(hs + NB * max_chunk);               // [max_chunk]
    for (int k = tid; k < nwords; k += FUSED_THREADS)
        mw[k] = __hip_atomic_load(maskbuf + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const int wpl = (nwords + 63) / 64;
    int lane_first, n;
    {
        int c = 0;
        for (int j = 0; j < wpl; ++j) {
            const int k = lane * wpl + j;
            if (k < nwords) c += __popcll(mw[k]);
        }
        const int inc = wave_inclusive_scan(c);
        lane_first = inc - c;
        n = __builtin_amdgcn_readlane(inc, 63);
    }
    const int chunk = chunk_of(n, G);
    const int lo = min(n, bid * chunk), hi = min(n, lo + chunk);
    const int cnt = hi - lo;
    const int gact = n > 0 ? (n + chunk - 1) / chunk : 0;
    if (bid == 0 && tid == 0 && nnz_out != nullptr) *nnz_out = n;

    if (cnt > 0) {
        const int ngroups = (cnt + UB - 1) / UB, padded = ngroups * UB;
        if (wave == 0) {
            int p = lane_first;
            for (int j = 0; j < wpl; ++j) {
                const int k = lane * wpl + j;
                const uint64_t w = k < nwords ? mw[k] : 0ull;
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
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if (lane < padded - cnt) lidx[cnt + lane] = lidx[cnt - 1];
        }
        for (int i = cnt + tid; i < padded; i += FUSED_THREADS)
#pragma unroll
            for (int b = 0; b < NB; ++b) hs[b * max_chunk + i] = 0.f;
        __syncthreads();
        if (idx_out != nullptr)
            for (int q = tid; q < cnt; q += FUSED_THREADS) idx_out[lo + q] = lidx[q];

        const bool drelu = (flags & 1u) != 0;
        const bool revalidate = (flags & 2u) != 0;
        const int nhv = d / HV;                       // 8-byte column groups of a row
        // first group of W_downT rows for this thread's first column group
        uint2 cur[UB];
        const bool preload = !revalidate && tid < nhv;
        if (preload) {
#pragma unroll
            for (int k = 0; k < UB; ++k)
                cur[k] = *reinterpret_cast<const uint2 *>(WdT + (size_t)lidx[k] * d + (size_t)tid * HV);
        }
        // ---- gate and up: one wave per row ----
        const int nfull = nvec / (64 * UA);
        for (int q = wave; q < cnt; q += FUSED_WAVES) {
            const size_t row = (size_t)lidx[q];
            const W *g = Wg + row * d + (size_t)lane * VEC;
            const W *u = Wu + row * d + (size_t)lane * VEC;
            float ag[NB], au[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) ag[b] = au[b] = 0.f;
            for (int it = 0; it < nfull; ++it) {
                uint4 rg[UA], ru[UA];
#pragma unroll
                for (int k = 0; k < UA; ++k) {
                    rg[k] = load_raw(g + (size_t)(it * UA + k) * 64 * VEC);
                    ru[k] = load_raw(u + (size_t)(it * UA + k) * 64 * VEC);
                }
#pragma unroll
                for (int k = 0; k < UA; ++k) {
                    const int v = lane + (it * UA + k) * 64;
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        const uint4 xv = xraw[b * nvec + v];
                        ag[b] = dot_raw(rg[k], xv, ag[b], (const W *)nullptr);
                        au[b] = dot_raw(ru[k], xv, au[b], (const W *)nullptr);
                    }
                }
            }
            for (int v = lane + nfull * UA * 64; v < nvec; v += 64) {
                const uint4 rg = load_raw(Wg + row * d + (size_t)v * VEC);
                const uint4 ru = load_raw(Wu + row * d + (size_t)v * VEC);
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const uint4 xv = xraw[b * nvec + v];
                    ag[b] = dot_raw(rg, xv, ag[b], (const W *)nullptr);
                    au[b] = dot_raw(ru, xv, au[b], (const W *)nullptr);
                }
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const float gs = wave_sum(ag[b]);
                const float us = wave_sum(au[b]);
                if (lane == 0) {
                    const float gp = fmaxf(gs, 0.f);
                    const float uu = drelu ? fmaxf(us, 0.f) : us;
                    hs[b * max_chunk + q] = gp * uu;
                }
            }
        }
        __syncthreads();
        // ---- down: every thread owns 8-byte column groups of the output ----
        for (int v = tid; v < nhv; v += FUSED_THREADS) {
            float acc[NB][HV];
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int e = 0; e < HV; ++e) acc[b][e] = 0.f;
            const W *colp = WdT + (size_t)v * HV;
            if (revalidate) {
                for (int q = 0; q < cnt; ++q) {
                    float h[NB];
                    bool any = false;
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        h[b] = hs[b * max_chunk + q];
                        any = any || (h[b] != 0.f);
                    }
                    if (!any) continue;
                    float w[HV];
                    widen_half(*reinterpret_cast<const uint2 *>(colp + (size_t)lidx[q] * d), w, (const W *)nullptr);
#pragma unroll
                    for (int b = 0; b < NB; ++b)
#pragma unroll
                        for (int e = 0; e < HV; ++e) acc[b][e] = fmaf(h[b], w[e], acc[b][e]);
                }
            } else {
                if (v != tid) {
#pragma unroll
                    for (int k = 0; k < UB; ++k)
                        cur[k] = *reinterpret_cast<const uint2 *>(colp + (size_t)lidx[k] * d);
                }
                for (int gq = 0; gq < ngroups; ++gq) {
                    uint2 nxt[UB];
                    if (gq + 1 < ngroups) {
#pragma unroll
                        for (int k = 0; k < UB; ++k)
                            nxt[k] = *reinterpret_cast<const uint2 *>(colp + (size_t)lidx[(gq + 1) * UB + k] * d);
                    }
#pragma unroll
                    for (int k = 0; k < UB; ++k) {
                        float w[HV];
                        widen_half(cur[k], w, (const W *)nullptr);
#pragma unroll
                        for (int b = 0; b < NB; ++b) {
                            const float h = hs[b * max_chunk + gq * UB + k];
#pragma unroll
                            for (int e = 0; e < HV; ++e) acc[b][e] = fmaf(h, w[e], acc[b][e]);
                        }
                    }
#pragma unroll
                    for (int k = 0; k < UB; ++k) cur[k] = nxt[k];
                }
            }
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int e = 0; e < HV; ++e)
                    store_wt(ypart + ((size_t)bid * NB + b) * d + (size_t)v * HV + e, acc[b][e]);
        }
        wait_stores_done();
    }
    __syncthreads();
    if (tid == 0) signal(ctrl, CTRL_Y, bid);
    SVDP_STAMP(0, 5);

    // ================= stage 4: y = sum of the partial y's, a slice of columns per block =================
    wait_stage(ctrl, CTRL_Y, G, spin_limit);
    SVDP_STAMP(0, 6);
    {
        float4 *red = reinterpret_cast<float4 *>(scratch);          // [256][4]
        const int c = tid & 3, seg = tid >> 2;                      // 4 float4 columns x 256 partials
        const int ncolq = (d / 4 + 3) / 4;
        for (int cb = bid; cb < ncolq; cb += G) {
            const int v = cb * 4 + c;                               // float4 column
            for (int b = 0; b < B; ++b) {
                float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
                if (v < d / 4) {
                    for (int g = seg; g < gact; g += FUSED_THREADS / 4) {
                        const float4 p = load_wt4(ypart + ((size_t)g * NB + b) * d + (size_t)v * 4);
                        s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
                    }
                }
                red[seg * 4 + c] = s;
                __syncthreads();
                for (int width = 64; width >= 1; width /= 4) {
                    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (seg < width) {
                        t = red[(4 * seg) * 4 + c];
#pragma unroll
                        for (int q = 1; q < 4; ++q) {
                            const float4 p = red[(4 * seg + q) * 4 + c];
                            t.x += p.x; t.y += p.y; t.z += p.z; t.w += p.w;
                        }
                    }
                    __syncthreads();
                    if (seg < width) red[seg * 4 + c] = t;
                    __syncthreads();
                }
                if (seg == 0 && v < d / 4) reinterpret_cast<float4 *>(y)[(size_t)b * (d / 4) + v] = red[c];
                __syncthreads();
            }
        }
    }

    SVDP_STAMP(0, 7);
    // ================= leave: the last block zeroes the counters =================
    if (tid == 0) {
        wait_stores_done();          // this thread's signals have been performed before it reports leaving
        const uint32_t old = __hip_atomic_fetch_add(ctrl + CTRL_EXIT, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old == (uint32_t)G - 1u) {
            for (int c = 0; c < 3 * CTRL_GROUPS; ++c)
                __hip_atomic_store(ctrl + c * CTRL_STRIDE, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(ctrl + CTRL_EXIT, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

}  // namespace svdp
