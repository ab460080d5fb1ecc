// Row kernel of the SEQUENTIAL pipeline (Sec. 4.2: the gate output re-validates
// the predictor's mask before the up and down projections are touched; Alg. 3's
// SparseUpAndMul and SparseDown test the gate result, not the predicted mask).
// Same contract, list handling, chunking and partial-y layout as k_rows; the
// phases differ:
//   phase G: one wave per listed row: g = W_gate[i].x for every token; only if
//            some token has g > 0 (a wave-uniform test) the row of W_up is
//            fetched and h = ReLU(g)*u formed; other rows end here;
//   then     wave 0 compacts the surviving rows of the chunk (ballot + popcount),
//            and their h and indices are packed;
//   phase B: as in k_rows, over the survivors only, so rows of W_downT whose
//            gate was <= 0 for every token are never read.
// Dropped terms are exact zeros, so y has the values of the parallel pipeline.
// Bytes read per listed row: d*w for the gate, 2*d*w more only if it survives.
// Dynamic LDS: NB*d storage elements (x) + 2*NB*max_chunk floats (h, packed h)
// + 3*max_chunk ints (list, flags / packed rows, survivor positions).
#pragma once

#include "svdp_kernels.h"

namespace svdp {

template <typename W, int NB, int MODE>
__global__ __launch_bounds__(ROWS_THREADS) __attribute__((amdgpu_waves_per_eu(4))) void k_rows_seq(
    const W *__restrict__ Wg, const W *__restrict__ Wu, const W *__restrict__ WdT, const W *__restrict__ x, int B,
    int d, int D, const uint64_t *__restrict__ mask, const int32_t *__restrict__ idx_in,
    const int32_t *__restrict__ nnz_in, int32_t *__restrict__ idx_out, int32_t *__restrict__ nnz_out,
    int32_t *__restrict__ n_used, int max_chunk, int min_chunk, uint32_t flags, float *__restrict__ ypart)
{
    constexpr int VEC = Elem<W>::VEC;
    constexpr int UG = NB <= 2 ? 8 : 4;     // 16-byte loads of one matrix in flight per lane in phase G
    constexpr int UB = 4;                   // rows of W_downT per group in phase B
    extern __shared__ uint4 smem16[];
    __shared__ int ns_shared;
    const int nvec = d / VEC;
    uint4 *xraw = smem16;                                        // [NB][nvec] x in storage form
    float *hs = reinterpret_cast<float *>(xraw + NB * nvec);     // [NB][max_chunk] by list position
    float *hp = hs + NB * max_chunk;                             // [NB][max_chunk] packed: survivors only
    int *lidx = reinterpret_cast<int *>(hp + NB * max_chunk);    // [max_chunk]
    int *srow = lidx + max_chunk;                                // [max_chunk] alive flags in phase G, then the survivors' rows
    int *spos = srow + max_chunk;                                // [max_chunk] list positions of the survivors
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int G = gridDim.x;

    uint4 xfirst[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
        xfirst[b] = (b < B && tid < nvec) ? load_raw(x + (size_t)b * d + (size_t)tid * VEC) : make_uint4(0u, 0u, 0u, 0u);
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

    rows_block_list<MODE>(D, mask, idx_in, lane_first, wpl, held, lo, hi, lidx);
    if (MODE == ROWS_MASK && idx_out != nullptr)
        for (int q = tid; q < cnt; q += ROWS_THREADS) idx_out[lo + q] = lidx[q];
    const bool drelu = (flags & 1u) != 0;

    // ---- phase G: gate, then up only where the gate is positive for some token.  A wave works on two
    // rows at a time (q and q + ROWS_WAVES) so that twice the loads are in flight ----
    auto row_dot2 = [&](const W *rowa, const W *rowb, bool has_b, float (&acca)[NB], float (&accb)[NB]) {
#pragma unroll
        for (int b = 0; b < NB; ++b) acca[b] = accb[b] = 0.f;
        const int nfull = nvec / (64 * UG);
        for (int it = 0; it < nfull; ++it) {
            uint4 ra[UG], rb[UG];
#pragma unroll
            for (int k = 0; k < UG; ++k) {
                ra[k] = load_raw(rowa + (size_t)(lane + (it * UG + k) * 64) * VEC);
                if (has_b) rb[k] = load_raw(rowb + (size_t)(lane + (it * UG + k) * 64) * VEC);
            }
#pragma unroll
            for (int k = 0; k < UG; ++k) {
                const int v = lane + (it * UG + k) * 64;
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const uint4 xv = xraw[b * nvec + v];
                    acca[b] = dot_raw(ra[k], xv, acca[b], (const W *)nullptr);
                    if (has_b) accb[b] = dot_raw(rb[k], xv, accb[b], (const W *)nullptr);
                }
            }
        }
        for (int v = lane + nfull * UG * 64; v < nvec; v += 64) {
            const uint4 ra = load_raw(rowa + (size_t)v * VEC);
            uint4 rb = ra;
            if (has_b) rb = load_raw(rowb + (size_t)v * VEC);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const uint4 xv = xraw[b * nvec + v];
                acca[b] = dot_raw(ra, xv, acca[b], (const W *)nullptr);
                if (has_b) accb[b] = dot_raw(rb, xv, accb[b], (const W *)nullptr);
            }
        }
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            acca[b] = wave_sum(acca[b]);
            accb[b] = wave_sum(accb[b]);
        }
    };
    for (int q = wave; q < cnt; q += 2 * ROWS_WAVES) {
        const int q2 = q + ROWS_WAVES;
        const bool two = q2 < cnt;                               // uniform over the wave
        // a rejected entry of the caller's list (-1) reads row 0 in its place and never survives
        const int ia = lidx[q], ib = lidx[two ? q2 : q];
        const size_t rowa = (size_t)max(ia, 0), rowb = (size_t)max(ib, 0);
        float ga[NB], gb[NB], ua[NB], ub[NB];
        row_dot2(Wg + rowa * d, Wg + rowb * d, two, ga, gb);
        bool alive_a = false, alive_b = false;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            alive_a = alive_a || (ia >= 0 && b < B && ga[b] > 0.f);
            alive_b = alive_b || (two && ib >= 0 && b < B && gb[b] > 0.f);
        }
        // both tests are uniform over the wave: the gates are wave sums
        if (alive_a && alive_b) {
            row_dot2(Wu + rowa * d, Wu + rowb * d, true, ua, ub);
        } else if (alive_a) {
            row_dot2(Wu + rowa * d, Wu + rowa * d, false, ua, ub);
        } else if (alive_b) {
            row_dot2(Wu + rowb * d, Wu + rowb * d, false, ub, ua);
        }
        if (lane == 0) {
            if (alive_a) {
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    hs[b * max_chunk + q] = fmaxf(ga[b], 0.f) * (drelu ? fmaxf(ua[b], 0.f) : ua[b]);
            }
            if (alive_b) {
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    hs[b * max_chunk + q2] = fmaxf(gb[b], 0.f) * (drelu ? fmaxf(ub[b], 0.f) : ub[b]);
            }
            srow[q] = alive_a ? 1 : 0;
            if (two) srow[q2] = alive_b ? 1 : 0;
        }
    }
    __syncthreads();

    // ---- survivors of the chunk, in list order ----
    if (wave == 0) {
        int run = 0;
        for (int base = 0; base < cnt; base += 64) {
            const int q = base + lane;
            const bool on = q < cnt && srow[q] != 0;
            const uint64_t bal = __ballot(on);
            if (on) spos[run + __popcll(bal & ((1ull << lane) - 1ull))] = q;
            run += __popcll(bal);
        }
        if (lane == 0) ns_shared = run;
    }
    __syncthreads();
    const int ns = ns_shared;
    const int ngroups = (ns + UB - 1) / UB;
    const int padded = ngroups * UB;
    // pack h and rows of the survivors; the last group is padded with repeats of the last row and h = 0
    for (int j = tid; j < padded; j += ROWS_THREADS) {
        const int q = spos[min(j, ns - 1)];
        srow[j] = lidx[q];
#pragma unroll
        for (int b = 0; b < NB; ++b) hp[b * max_chunk + j] = j < ns ? hs[b * max_chunk + q] : 0.f;
    }
    __syncthreads();

    // ---- phase B over the survivors (as in k_rows) ----
    for (int v = tid; v < nvec; v += ROWS_THREADS) {
        float acc[NB][VEC];
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[b][e] = 0.f;
        const W *colp = WdT + (size_t)v * VEC;
        uint4 cur[UB];
        if (ngroups > 0) {
#pragma unroll
            for (int k = 0; k < UB; ++k) cur[k] = load_raw(colp + (size_t)srow[k] * d);
        }
        for (int gq = 0; gq < ngroups; ++gq) {
            uint4 nxt[UB];
            if (gq + 1 < ngroups) {
#pragma unroll
                for (int k = 0; k < UB; ++k) nxt[k] = load_raw(colp + (size_t)srow[(gq + 1) * UB + k] * d);
            }
#pragma unroll
            for (int k = 0; k < UB; ++k) {
                float w[VEC];
                widen(cur[k], w, (const W *)nullptr);
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const float h = hp[b * max_chunk + gq * UB + k];
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

}   // namespace svdp
