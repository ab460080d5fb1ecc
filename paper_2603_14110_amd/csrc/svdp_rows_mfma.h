// Kernels on the matrix cores.
//
// The FFN over a list of rows for batches of several tokens in bf16 storage (the regime the paper's
// Sec. 6 names as the limit of the sparse path: the union of the tokens' masks is dense enough that a
// row-at-a-time kernel spends its time in per-token vector arithmetic, and App. C's Alg. 4 treats the
// selected rows as a small dense contraction), in two kernels:
//   k_gate_up_mfma  same contract and list handling as k_rows, but it ends with h = ReLU(g) * u of its
//            chunk of the list written to memory (h [list position][NB], and the checked list).  Tiles of 16
//            list rows x 64 elements of d; four lanes fetch 64 contiguous bytes of one row per load, two
//            loads cover 128 bytes and feed two v_mfma_f32_16x16x32_bf16 per matrix, whose other operand is
//            x in LDS, stored in operand order.  The eight waves of the block split d between them; their
//            16x16 partial tiles meet in LDS and are added in wave order.
//   k_down_slices   y[token][col] = sum over the list of h * W_downT[row][col], by blocks that own a
//            128-byte column slice and one of eight parts of the list (see there).
// Products of bf16 values are exact in fp32 and every sum has a fixed order.
// Requirements checked by the host: d % 512 == 0, NB <= 8.
// Dynamic LDS of k_gate_up_mfma: NB*d*2 bytes (x) + ROWS_WAVES*max_chunk*2*NB floats (partial tiles) +
// max_chunk ints (list); max_chunk % 16 == 0.
#pragma once

#include "svdp_kernels.h"

namespace svdp {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

constexpr int MF_ROWS = 16;      // list rows per tile
constexpr int MF_UA = 4;         // 64-element steps fetched together

__device__ __forceinline__ f32x4_t mfma_bf16(const uint4 &a, const uint4 &b, f32x4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                   0, 0, 0);
}

template <int NB, int MODE>
__global__ __launch_bounds__(ROWS_THREADS) void k_gate_up_mfma(
    const bf16 *__restrict__ Wg, const bf16 *__restrict__ Wu, const bf16 *__restrict__ x, int B, int d, int D,
    const uint64_t *__restrict__ mask, const int32_t *__restrict__ idx_in, const int32_t *__restrict__ nnz_in,
    int32_t *__restrict__ idx_out, int32_t *__restrict__ nnz_out, int32_t *__restrict__ n_used, int max_chunk,
    int min_chunk, uint32_t flags, float *__restrict__ hbuf, int32_t *__restrict__ lst)
{
    static_assert(NB == 1 || NB == 2 || NB == 4 || NB == 8, "token slots are addressed with a mask");
    extern __shared__ uint4 smem16[];
    const int nvec = d / 8;                                        // 16-byte vectors per token
    const int nsteps = d / 64;                                     // 64-element steps per row
    uint4 *xs = smem16;                                            // [nsteps][2][4][NB], operand order
    float *part = reinterpret_cast<float *>(xs + NB * nvec);       // [ROWS_WAVES][tiles][2][16][NB]
    int *lidx = reinterpret_cast<int *>(part + (size_t)ROWS_WAVES * max_chunk * 2 * NB);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lm = lane & 15, lq = lane >> 4;
    const int G = gridDim.x;

    // ---- request x; the vector of element 8c..8c+7 goes where the lane that needs it as an
    // operand will read it: step c/8, instruction (c/4)%2, lane quarter c%4, token ----
    auto xslot = [&](int c, int b) -> int { return (((c >> 3) * 2 + ((c >> 2) & 1)) * 4 + (c & 3)) * NB + b; };
    uint4 xfirst[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
        xfirst[b] = (b < B && tid < nvec) ? load_raw(x + (size_t)b * d + (size_t)tid * 8) : make_uint4(0u, 0u, 0u, 0u);

    int lane_first, wpl;
    uint64_t held[ROWS_WREG];
    const int n = rows_list_length<MODE>(D, mask, nnz_in, lane, lane_first, wpl, held);
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (tid < nvec) xs[xslot(tid, b)] = xfirst[b];
        for (int c = tid + ROWS_THREADS; c < nvec; c += ROWS_THREADS)
            xs[xslot(c, b)] = b < B ? load_raw(x + (size_t)b * d + (size_t)c * 8) : make_uint4(0u, 0u, 0u, 0u);
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
    if (MODE != ROWS_DENSE)
        for (int q = tid; q < cnt; q += ROWS_THREADS) lst[lo + q] = lidx[q];

    const bool drelu = (flags & 1u) != 0;
    // rows past the end of the chunk repeat its last row, and a rejected entry of the caller's list
    // (-1) reads row 0 in its place; the h of both is zero
    auto row_of = [&](int q) -> size_t {
        const int qq = min(q, cnt - 1);
        return MODE == ROWS_DENSE ? (size_t)(lo + qq) : (size_t)max(lidx[qq], 0);
    };
    const int ntile = (cnt + MF_ROWS - 1) / MF_ROWS;

    // ---- this wave's share of d is the steps [wave*spw, (wave+1)*spw) ----
    const int spw = nsteps / ROWS_WAVES;
    const int tb = lm & (NB - 1);                                   // token slot read as the x operand
    for (int t = 0; t < ntile; ++t) {
        const size_t row = row_of(t * MF_ROWS + lm);
        const bf16 *pg = Wg + row * d + (size_t)wave * spw * 64 + lq * 8;
        const bf16 *pu = Wu + row * d + (size_t)wave * spw * 64 + lq * 8;
        f32x4_t ag = {0.f, 0.f, 0.f, 0.f}, au = {0.f, 0.f, 0.f, 0.f};
        for (int s0 = 0; s0 < spw; s0 += MF_UA) {
            uint4 g0[MF_UA], g1[MF_UA], u0[MF_UA], u1[MF_UA];
#pragma unroll
            for (int k = 0; k < MF_UA; ++k) {
                if (s0 + k < spw) {
                    g0[k] = load_raw(pg + (size_t)(s0 + k) * 64);
                    g1[k] = load_raw(pg + (size_t)(s0 + k) * 64 + 32);
                    u0[k] = load_raw(pu + (size_t)(s0 + k) * 64);
                    u1[k] = load_raw(pu + (size_t)(s0 + k) * 64 + 32);
                }
            }
#pragma unroll
            for (int k = 0; k < MF_UA; ++k) {
                if (s0 + k < spw) {
                    const int s = wave * spw + s0 + k;
                    const uint4 xa = xs[((s * 2 + 0) * 4 + lq) * NB + tb];
                    const uint4 xb = xs[((s * 2 + 1) * 4 + lq) * NB + tb];
                    ag = mfma_bf16(g0[k], xa, ag);
                    au = mfma_bf16(u0[k], xa, au);
                    ag = mfma_bf16(g1[k], xb, ag);
                    au = mfma_bf16(u1[k], xb, au);
                }
            }
        }
        // the lane holds rows 4*lq .. 4*lq+3 of the tile for token lm
        if (lm < NB) {
            float *pt = part + ((size_t)(wave * ntile + t) * 2) * MF_ROWS * NB;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                pt[(lq * 4 + i) * NB + lm] = ag[i];
                pt[MF_ROWS * NB + (lq * 4 + i) * NB + lm] = au[i];
            }
        }
    }
    __syncthreads();
    // partial tiles of the waves, added in wave order -> h[list position][token]
    for (int e = tid; e < cnt * NB; e += ROWS_THREADS) {
        const int q = e / NB, b = e % NB;
        float h = 0.f;
        if (MODE != ROWS_LIST || lidx[q] >= 0) {
            const int t = q / MF_ROWS, rr = q % MF_ROWS;
            float gs = 0.f, us = 0.f;
#pragma unroll
            for (int w = 0; w < ROWS_WAVES; ++w) {
                const float *pt = part + ((size_t)(w * ntile + t) * 2) * MF_ROWS * NB;
                gs += pt[rr * NB + b];
                us += pt[MF_ROWS * NB + rr * NB + b];
            }
            h = fmaxf(gs, 0.f) * (drelu ? fmaxf(us, 0.f) : us);
        }
        hbuf[(size_t)(lo + q) * NB + b] = h;
    }
}

// ---------------------------------------------------------------------------
// Down projection over column slices, for batches (Alg. 4's last product; App. C: W_down is stored by columns,
// W_downT [D][d], so that a selected neuron is one contiguous row):
//     y[token][col] = sum over the list of h[position][token] * W_downT[row(position)][col].
// Block (slice, rg) owns the 64 columns (one 128-byte line of every row) [64 slice, +64) and the rg-th of RG equal
// parts of the list, and writes its sums to ypart [rg][NB][d]; k_reduce_y adds the RG parts.  Against one partial
// y per row-kernel block (256 of them: 32 MB written and read again at eight tokens) this leaves RG * NB * d
// floats.  Eight lanes fetch the 128 bytes of a row, so a wave's load instruction covers eight rows; a lane keeps
// NB x 8 sums (its eight columns for every token), and h (written by the gate/up kernel, a few hundred KB that stay
// in L2) is read by position.  The sums over a wave's eight row lanes and then over the waves are taken in a fixed
// order through LDS.
// Requirements checked by the host: d a multiple of the slice width, ceil(D / RG) <= DS_MAX_CHUNK.
// ---------------------------------------------------------------------------
constexpr int DS_THREADS = 256;
constexpr int DS_WAVES = DS_THREADS / 64;
constexpr int DS_UB = 4;             // wave loads (eight rows each) in flight, twice while the next group is fetched
constexpr int DS_MAX_CHUNK = 4096;   // list entries of a block kept in LDS
constexpr int DS_LPR = 8;            // lanes per row: 16 bytes each, one 128-byte line
constexpr int DS_SW = DS_LPR * 8;    // columns of a slice

template <int NB, bool DENSE>
__global__ __launch_bounds__(DS_THREADS) void k_down_slices(const bf16 *__restrict__ WdT,
                                                            const int32_t *__restrict__ lst,
                                                            const int32_t *__restrict__ n_ptr, int n_fixed, int D, int d,
                                                            const float *__restrict__ hbuf, int min_chunk,
                                                            float *__restrict__ ypart)
{
    constexpr int LPR = DS_LPR, SW = DS_SW;
    constexpr int RPW = 64 / LPR;                // rows per wave load
    constexpr int RSETS = RPW / 2;               // row-lane sets of a wave left after the lane shift below
    __shared__ int lidx[DENSE ? 1 : DS_MAX_CHUNK];
    __shared__ float red[DS_WAVES * RSETS * NB * SW];         // [DS_WAVES * RSETS][NB][SW]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int cg = lane % LPR, sub = lane / LPR;
    const int slice = blockIdx.x, rg = blockIdx.y, RG = gridDim.y;
    int n = n_ptr != nullptr ? *n_ptr : n_fixed;
    n = max(0, min(n, D));
    const int chunk = chunk_of(n, RG, min_chunk);
    const int lo = min(n, rg * chunk), hi = min(n, lo + chunk), cnt = hi - lo;
    if (cnt <= 0) return;
    if (!DENSE) {
        for (int q = tid; q < cnt; q += DS_THREADS) lidx[q] = lst[lo + q];
        __syncthreads();
    }
    const bf16 *colp = WdT + (size_t)slice * SW + (size_t)cg * 8;
    const int ngroups = (cnt + RPW - 1) / RPW;

    // v_mfma_f32_4x4x1_16b: sixteen independent 4 x 4 outer products; the four lanes of a block work on the same
    // row, lane j of the block supplies h of token 4 tg + j and its own column's weight, and keeps the four tokens'
    // sums for its own column: acc[tg][e][i] belongs to token 4 tg + i and column 8 cg + e.
    constexpr int TG = (NB + 3) / 4;
    f32x4_t acc[TG][8];
#pragma unroll
    for (int g = 0; g < TG; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // group g of the chunk = its rows RPW g .. RPW g + RPW - 1; this wave takes the groups wave, wave + DS_WAVES, ...
    auto fetch = [&](int g0, uint4 (&wv)[DS_UB], float (&hv)[DS_UB][TG]) {
#pragma unroll
        for (int k = 0; k < DS_UB; ++k) {
            const int q = (g0 + k * DS_WAVES) * RPW + sub;
            wv[k] = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int g = 0; g < TG; ++g) hv[k][g] = 0.f;
            if (q < cnt) {
                const int row = DENSE ? lo + q : lidx[q];
                if (row >= 0) {                                    // a rejected entry of the caller's list: h is zero
                    wv[k] = load_raw(colp + (size_t)row * d);
                    const float *hp = hbuf + (size_t)(lo + q) * NB;
#pragma unroll
                    for (int g = 0; g < TG; ++g)
                        if (g * 4 + (lane & 3) < NB) hv[k][g] = hp[g * 4 + (lane & 3)];
                }
            }
        }
    };
    auto consume = [&](const uint4 (&wv)[DS_UB], const float (&hv)[DS_UB][TG]) {
#pragma unroll
        for (int k = 0; k < DS_UB; ++k) {
            float w[8];
            widen(wv[k], w, (const bf16 *)nullptr);
#pragma unroll
            for (int e = 0; e < 8; ++e)
#pragma unroll
                for (int g = 0; g < TG; ++g)
                    acc[g][e] = __builtin_amdgcn_mfma_f32_4x4x1f32(hv[k][g], w[e], acc[g][e], 0, 0, 0);
        }
    };
    {
        uint4 wa[DS_UB], wb[DS_UB];
        float ha[DS_UB][TG], hb[DS_UB][TG];
        constexpr int STEP = DS_WAVES * DS_UB;
        fetch(wave, wa, ha);
        for (int g0 = wave; g0 < ngroups; g0 += 2 * STEP) {
            fetch(g0 + STEP, wb, hb);            // past the end: nothing is requested
            consume(wa, ha);
            fetch(g0 + 2 * STEP, wa, ha);
            consume(wb, hb);
        }
    }
    // row lanes l and l ^ 8 first (a lane shift), then the four remaining sets of a wave and the waves through
    // LDS, in order
#pragma unroll
    for (int g = 0; g < TG; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[g][e][i] += dpp_move<0x128>(acc[g][e][i]);           // row_ror:8
    if ((sub & 1) == 0) {
        const int set = wave * RSETS + (sub >> 1);
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int e = 0; e < 8; ++e) red[(set * NB + b) * SW + cg * 8 + e] = acc[b / 4][e][b % 4];
    }
    __syncthreads();
    for (int o = tid; o < NB * SW; o += DS_THREADS) {
        const int b = o / SW, c = o % SW;
        float t = 0.f;
#pragma unroll
        for (int p = 0; p < DS_WAVES * RSETS; ++p) t += red[(p * NB + b) * SW + c];
        ypart[((size_t)rg * NB + b) * d + (size_t)slice * SW + c] = t;
    }
}

// ---------------------------------------------------------------------------
// Predictor stage 2 on the matrix cores: s_i = t . Q[i,:] + b_i for a slab of
// 64 neurons and up to eight tokens, and the slab's mask word (eq. 2).  One
// wave per 16 rows of Q; a lane fetches 16 bytes of one row per 32 columns
// (all requested before t is touched).  t (fp32, the sum of the nt stage-1
// partials) is split into three bf16 terms hi + mid + lo = t exactly to 24 bits,
// stored in LDS in operand order, so that bf16 MFMAs give fp32-accurate scores:
// every product is exact and the accumulation is fp32.
// Requirements checked by the host: r % 32 == 0, r <= 32 * SCM_KB.
// Dynamic LDS: 3 * NB * r * 2 bytes.
// ---------------------------------------------------------------------------
constexpr int SCM_THREADS = 256;
constexpr int SCM_KB = 16;          // 32-column blocks of Q held in registers

__device__ __forceinline__ uint32_t bf16_rne_bits(float v)
{
    bf16 h;
    from_f32(v, &h);
    return h.bits;
}

template <int NB>
__global__ __launch_bounds__(SCM_THREADS) void k_scores_mfma(const bf16 *__restrict__ Q, const float *__restrict__ bias,
                                                             const float *__restrict__ tpart, int nt, int B, int D,
                                                             int r, float *__restrict__ s_out,
                                                             uint64_t *__restrict__ mask_out)
{
    static_assert(NB == 1 || NB == 2 || NB == 4 || NB == 8, "token slots are addressed with a mask");
    extern __shared__ uint4 smem16[];
    __shared__ uint32_t word16[SCM_THREADS / 64];
    uint4 *planes = smem16;                                         // [3][r/32][4][NB]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lm = lane & 15, lq = lane >> 4;
    const int i0 = blockIdx.x * SC_SLAB + wave * 16;
    const int nkb = r / 32;

    uint4 q[SCM_KB];
    const bf16 *qrow = Q + (size_t)(i0 + lm) * r + lq * 8;
#pragma unroll
    for (int kb = 0; kb < SCM_KB; ++kb)
        if (kb < nkb) q[kb] = load_raw(qrow + kb * 32);
    const float4 bs = *reinterpret_cast<const float4 *>(bias + i0 + lq * 4);

    // t for (token b, columns 8g .. 8g+7): sum of the partials in order, then the three terms
    const int ngr = r / 8;
    for (int u = tid; u < NB * ngr; u += SCM_THREADS) {
        const int b = u / ngr, g = u % ngr;
        float t[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) t[e] = 0.f;
        const float4 *tp = reinterpret_cast<const float4 *>(tpart + (size_t)b * r + (size_t)g * 8);
        const size_t stride4 = (size_t)NB * r / 4;
#pragma unroll 4
        for (int p = 0; p < nt; ++p) {
            const float4 a = tp[p * stride4], c = tp[p * stride4 + 1];
            t[0] += a.x; t[1] += a.y; t[2] += a.z; t[3] += a.w;
            t[4] += c.x; t[5] += c.y; t[6] += c.z; t[7] += c.w;
        }
        uint32_t pl[3][8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t hi = bf16_rne_bits(t[e]);
            const float r1 = t[e] - __uint_as_float(hi << 16);
            const uint32_t mid = bf16_rne_bits(r1);
            const float r2 = r1 - __uint_as_float(mid << 16);
            pl[0][e] = hi; pl[1][e] = mid; pl[2][e] = bf16_rne_bits(r2);
        }
        const int slot = ((g >> 2) * 4 + (g & 3)) * NB + b;
#pragma unroll
        for (int p = 0; p < 3; ++p)
            planes[(size_t)p * nkb * 4 * NB + slot] =
                make_uint4(pl[p][0] | (pl[p][1] << 16), pl[p][2] | (pl[p][3] << 16), pl[p][4] | (pl[p][5] << 16),
                           pl[p][6] | (pl[p][7] << 16));
    }
    __syncthreads();

    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
    const int tb = lm & (NB - 1);
#pragma unroll
    for (int kb = 0; kb < SCM_KB; ++kb) {
        if (kb < nkb) {
#pragma unroll
            for (int p = 0; p < 3; ++p)
                acc = mfma_bf16(q[kb], planes[(size_t)p * nkb * 4 * NB + (kb * 4 + lq) * NB + tb], acc);
        }
    }
    // the lane holds rows i0 + 4*lq .. +3 for token lm
    const float sv[4] = {acc[0] + bs.x, acc[1] + bs.y, acc[2] + bs.z, acc[3] + bs.w};
    if (s_out != nullptr && lm < B) {
#pragma unroll
        for (int i = 0; i < 4; ++i) s_out[(size_t)lm * D + i0 + lq * 4 + i] = sv[i];
    }
    if (mask_out != nullptr) {
        uint32_t w16 = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint64_t on = __ballot(lm < B && sv[i] > 0.f);
#pragma unroll
            for (int qq = 0; qq < 4; ++qq)
                if ((on >> (16 * qq)) & 0xffffull) w16 |= 1u << (4 * qq + i);
        }
        if (lane == 0) word16[wave] = w16;
        __syncthreads();
        if (tid == 0)
            mask_out[blockIdx.x] = (uint64_t)word16[0] | ((uint64_t)word16[1] << 16) | ((uint64_t)word16[2] << 32) |
                                   ((uint64_t)word16[3] << 48);
    }
}

}   // namespace svdp
