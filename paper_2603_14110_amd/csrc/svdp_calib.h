// Offline bias calibration on the GPU (Alg. 2 of the paper, "Greedy Bias
// Calibration"; App. A "Greedy threshold selection"), from given damage weights
// w [D][T] and proxy scores s [D][T].
//
// The printed algorithm is a loop over a priority queue: pop the neuron whose
// next eta samples cost least, advance its pointer, push its next cost, until
// enough (neuron, sample) pairs are dropped.  That order has a closed form: a
// neuron's steps leave the queue in the order of the RUNNING MAXIMUM of its step
// costs (a step cheaper than its predecessor is taken right after it), so the
// whole sequence is all steps sorted by (running-max cost, neuron, step).  Two
// kernels follow from it:
//   k_calib_sort   one block per neuron: the samples from the first positive weight
//                  on (in the order by score, ties by sample index) are sorted
//                  in LDS, the ones below only counted; step costs (fp32, left
//                  to right), their running maxima, and for every step the
//                  number of dropped samples and the threshold it would set;
//                  optionally the Kendall check of App. A.
//   k_select_*     the cost level at which the required number of pairs is first
//                  reached, by a radix select over the keys' bit patterns
//                  (four digit passes, integer atomics); then one block takes
//                  the steps at exactly that level in neuron order and writes
//                  b = -tau and the pointers.
// Integer results equal the sequential algorithm's bit for bit.
#pragma once

#include "svdp_device.h"

namespace svdp {

constexpr int CAL_THREADS = 512;
constexpr int CAL_MAX_T = 4096;
constexpr int SEL_THREADS = 1024;

// order-preserving map float -> uint32 (-0 and +0 coincide; inputs are not NaN)
__device__ __forceinline__ uint32_t ordered_bits(float v)
{
    uint32_t u = __float_as_uint(v == 0.f ? 0.f : v);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Per-neuron tables written by k_calib_sort, MS = ceil(T / eta) steps at most:
//   key  [D][MS]     running maximum of the step costs, +inf beyond the neuron's last step
//   drop [D][MS + 1] number of samples with s <= tau after 0, 1, 2, ... steps
//   tauc [D][MS + 1] the threshold after 0, 1, 2, ... steps
//   k0   [D]         the starting pointer (1-based count)
// Only the part of the order that the algorithm walks is sorted: everything below the first sample
// with a positive weight (in the order by score, then sample index) is merely counted -- those
// samples have zero weight and are dropped from the start -- and the rest, the "tail", typically a
// tenth of the samples of a sparse layer, goes through a bitonic sort sized to it.
// Dynamic LDS: n2*8 (sort keys) + 2*T*4 (sorted tail: s, w) + 2*(MS+1)*4 bytes, n2 = T rounded up to a power of two.
__global__ __launch_bounds__(CAL_THREADS) void k_calib_sort(const float *__restrict__ w, const float *__restrict__ s,
                                                            int T, int n2max, int eta, int MS,
                                                            float *__restrict__ key, int32_t *__restrict__ drop,
                                                            float *__restrict__ tauc, int32_t *__restrict__ k0_out,
                                                            float *__restrict__ kendall)
{
    extern __shared__ unsigned long long smem64[];
    unsigned long long *sk = smem64;                               // [n2max]
    float *ss = reinterpret_cast<float *>(sk + n2max);             // [T] scores of the tail, sorted
    float *ww = ss + T;                                            // [T] weights in that order
    float *cost = ww + T;                                          // [MS + 1]
    float *scan = cost + (MS + 1);                                 // [MS + 1]
    __shared__ unsigned long long kmin_sh;                         // smallest (score, sample) key with a positive weight
    __shared__ unsigned long long kmax_sh;                         // largest (score, sample) key: the last sample in sorted order
    __shared__ int below_sh, fill_sh, kd_total;
    const int i = blockIdx.x, tid = threadIdx.x;
    const float *si = s + (size_t)i * T, *wi = w + (size_t)i * T;
    auto key_of = [&](int t) { return ((unsigned long long)ordered_bits(si[t]) << 32) | (unsigned)t; };

    if (tid == 0) {
        kmin_sh = ~0ull;
        kmax_sh = 0ull;
        below_sh = 0;
        fill_sh = 0;
        kd_total = 0;
    }
    __syncthreads();
    {
        unsigned long long kmin = ~0ull;
        unsigned long long kmax = 0ull;
        for (int t = tid; t < T; t += CAL_THREADS) {
            const unsigned long long k = key_of(t);
            if (wi[t] > 0.f && k < kmin) kmin = k;
            if (k > kmax) kmax = k;
        }
        if (kmin != ~0ull) atomicMin(&kmin_sh, kmin);
        atomicMax(&kmax_sh, kmax);
    }
    __syncthreads();
    const unsigned long long kmin = kmin_sh;
    // the tail: samples at or above the first positive one; the rest is counted
    {
        int below = 0;
        for (int t = tid; t < T; t += CAL_THREADS) {
            const unsigned long long k = key_of(t);
            if (k < kmin) ++below;
            else sk[atomicAdd(&fill_sh, 1)] = k;                   // any order: sorted next
        }
        if (below) atomicAdd(&below_sh, below);
    }
    __syncthreads();
    const int nb = below_sh;                                       // samples below the tail (T if no weight is positive)
    const int ntail = T - nb;
    int n2 = 1;
    while (n2 < ntail) n2 <<= 1;
    for (int t = ntail + tid; t < n2; t += CAL_THREADS) sk[t] = ~0ull;
    __syncthreads();
    for (int k = 2; k <= n2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = tid; t < n2; t += CAL_THREADS) {
                const int p = t ^ j;
                if (p > t) {
                    const unsigned long long a = sk[t], b = sk[p];
                    const bool up = (t & k) == 0;
                    if ((a > b) == up) {
                        sk[t] = b;
                        sk[p] = a;
                    }
                }
            }
            __syncthreads();
        }
    }
    for (int p = tid; p < ntail; p += CAL_THREADS) {
        const int t = (int)(sk[p] & 0xffffffffu);
        ss[p] = si[t];
        ww[p] = wi[t];
    }
    __syncthreads();
    // sorted position q of the whole sample = tail position q - nb; the first positive weight is tail position 0
    const int k0 = ntail > 0 ? nb + 1 : T;                         // min{k : w_(k) > 0}, or T if there is none
    const int M = (T - k0 + eta - 1) / eta;                        // steps this neuron can take

    // step costs C(k + eta) - C(k), fp32 left to right; the last step may be short (the listing's padding)
    for (int j = tid; j < M; j += CAL_THREADS) {
        const int lo = k0 - nb + j * eta, hi = min(lo + eta, ntail);
        float c = 0.f;
        for (int p = lo; p < hi; ++p) c += ww[p];
        cost[j] = c;
    }
    __syncthreads();
    // running maximum (inclusive), Hillis-Steele over M entries
    float *src = cost, *dst = scan;
    for (int off = 1; off < M; off <<= 1) {
        for (int j = tid; j < M; j += CAL_THREADS) dst[j] = j >= off ? fmaxf(src[j], src[j - off]) : src[j];
        __syncthreads();
        float *tmp = src;
        src = dst;
        dst = tmp;
    }
    for (int j = tid; j < MS; j += CAL_THREADS) key[(size_t)i * MS + j] = j < M ? src[j] : __builtin_inff();
    // thresholds and dropped counts after j steps: k = min(k0 + j*eta, T), tau = s_(k), #{s <= tau};
    // every sample below the tail has a score <= tau
    for (int j = tid; j <= MS; j += CAL_THREADS) {
        int dj = 0;
        float tj = 0.f;
        if (j <= M) {
            if (ntail == 0) {                                       // nothing ever active: all dropped, tau = the last score
                tj = si[(int)(kmax_sh & 0xffffffffu)];
                dj = T;
            } else {
                const int k = min(k0 + j * eta, T) - nb;            // tail count, >= 1
                tj = ss[k - 1];
                int lo = k, hi = ntail;                             // first tail position whose score exceeds tau
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (ss[mid] <= tj) lo = mid + 1;
                    else hi = mid;
                }
                dj = nb + lo;
            }
        }
        drop[(size_t)i * (MS + 1) + j] = dj;
        tauc[(size_t)i * (MS + 1) + j] = tj;
    }
    if (tid == 0) k0_out[i] = k0;

    if (kendall != nullptr) {
        // App. A: non-overlapping eta-step sums over the whole sorted sample (zero below the tail),
        // discordant pairs m1 < m2
        const int MK = T / eta;
        __syncthreads();                                            // cost/scan are free again
        float *S = cost;                                            // MK <= MS entries
        for (int m = tid; m < MK; m += CAL_THREADS) {
            float c = 0.f;
            for (int q = max(m * eta, nb); q < (m + 1) * eta; ++q) c += ww[q - nb];
            S[m] = c;
        }
        __syncthreads();
        int kd = 0;
        for (int m1 = tid; m1 < MK; m1 += CAL_THREADS) {
            const float a = S[m1];
            for (int m2 = m1 + 1; m2 < MK; ++m2) kd += a > S[m2] ? 1 : 0;
        }
        if (kd) atomicAdd(&kd_total, kd);
        __syncthreads();
        if (tid == 0) kendall[i] = MK < 2 ? 1.f : (float)(1.0 - (double)kd_total / ((double)MK * (MK - 1)));
    }
}

// Block-wide sum of a 64-bit count (every thread gets the result).
__device__ __forceinline__ long long block_sum_i64(long long v, long long *red)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();
    if (lane == 0) red[wave] = v;
    __syncthreads();
    long long t = 0;
    for (int q = 0; q < (int)blockDim.x / 64; ++q) t += red[q];
    return t;
}

// Number of steps of a neuron whose key is <= level (INCLUSIVE) or < level (keys are non-decreasing; +inf pads).
template <bool INCLUSIVE>
__device__ __forceinline__ int steps_below(const float *__restrict__ key_i, int MS, float level)
{
    int lo = 0, hi = MS;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        const float v = key_i[mid];
        if (INCLUSIVE ? v <= level : v < level) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

// The cost level at which the required number of pairs is first reached is found by a radix
// select over the bit patterns of the (non-negative) keys, most significant digit first: the pairs a
// step adds (its gain) are summed per digit value among the steps that match the digits found so
// far, and the digit is where the running sum first covers what is still missing.  Integer atomics
// only, so the result does not depend on the order of arrival.
struct SelectState {
    long long missing;       // pairs still to be found among steps at or above the current prefix
    long long c0;            // pairs dropped before any step
    uint32_t prefix;         // digits of the level found so far
    int32_t reachable;       // 0: the start already meets the target, or all finite steps together do not
    int32_t at_start;        // 1: the start already meets the target (no step is taken)
};
constexpr int SEL_BINS = 256;
constexpr uint32_t SEL_TOP = 0x7f7fffffu;      // largest finite float: keys above it are padding

__global__ __launch_bounds__(SEL_THREADS) void k_select_init(const int32_t *__restrict__ drop, int D, int MS,
                                                             long long need, SelectState *__restrict__ st,
                                                             long long *__restrict__ hist)
{
    __shared__ long long red[SEL_THREADS / 64];
    long long c0 = 0;
    for (int i = threadIdx.x; i < D; i += SEL_THREADS) c0 += drop[(size_t)i * (MS + 1)];
    c0 = block_sum_i64(c0, red);
    if (threadIdx.x < SEL_BINS) hist[threadIdx.x] = 0;
    if (threadIdx.x == 0) {
        st->c0 = c0;
        st->missing = need - c0;
        st->prefix = 0u;
        st->reachable = c0 < need ? 1 : 0;
        st->at_start = c0 < need ? 0 : 1;
    }
}

// hist[digit] += gain over the steps whose key matches the prefix above this digit.
template <int SHIFT, int BITS>
__global__ __launch_bounds__(256) void k_select_hist(const float *__restrict__ key, const int32_t *__restrict__ drop,
                                                     int D, int MS, const SelectState *__restrict__ st,
                                                     long long *__restrict__ hist)
{
    __shared__ long long lh[SEL_BINS];
    if (st->reachable == 0) return;
    const uint32_t prefix = st->prefix;
    for (int q = threadIdx.x; q < SEL_BINS; q += 256) lh[q] = 0;
    __syncthreads();
    const size_t total = (size_t)D * MS;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
        const int i = (int)(e / MS), j = (int)(e % MS);
        const uint32_t kb = __float_as_uint(key[e]);
        if (kb > SEL_TOP) continue;
        if (SHIFT + BITS < 31 && (kb >> (SHIFT + BITS)) != (prefix >> (SHIFT + BITS))) continue;
        const int32_t *di = drop + (size_t)i * (MS + 1);
        const long long gain = (long long)di[j + 1] - di[j];
        if (gain != 0) atomicAdd(reinterpret_cast<unsigned long long *>(&lh[(kb >> SHIFT) & ((1u << BITS) - 1u)]),
                                 (unsigned long long)gain);
    }
    __syncthreads();
    for (int q = threadIdx.x; q < SEL_BINS; q += 256)
        if (lh[q] != 0) atomicAdd(reinterpret_cast<unsigned long long *>(&hist[q]), (unsigned long long)lh[q]);
}

// Picks the digit, updates the state and clears the histogram for the next digit.  One wave:
// lane l owns bins 4l .. 4l+3, a shuffle scan gives the running sums.
template <int SHIFT, bool FIRST>
__global__ __launch_bounds__(64) void k_select_pick(SelectState *__restrict__ st, long long *__restrict__ hist)
{
    const int lane = threadIdx.x;
    long long h[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        h[q] = hist[4 * lane + q];
        hist[4 * lane + q] = 0;
    }
    if (st->reachable == 0) return;
    const long long missing = st->missing;
    const long long mine = h[0] + h[1] + h[2] + h[3];
    long long inc = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const long long o = __shfl_up(inc, off);
        if (lane >= off) inc += o;
    }
    const long long before = inc - mine;
    const bool here = before < missing && inc >= missing;           // at most one lane
    const unsigned long long who = __ballot(here);
    if (who == 0ull) {
        if (lane == 0) st->reachable = 0;       // only on the first digit: every finite step together falls short
        return;
    }
    if (here) {
        long long run = before;
        int digit = 0;
        for (int q = 0; q < 4; ++q) {
            if (run + h[q] >= missing) {
                digit = 4 * lane + q;
                break;
            }
            run += h[q];
        }
        st->missing = missing - run;            // still to be found among the steps with this digit
        st->prefix |= (uint32_t)digit << SHIFT;
    }
}

// With the level known, per neuron: the number of its steps strictly below the level and up to it.
__global__ __launch_bounds__(256) void k_select_bounds(const float *__restrict__ key, int D, int MS,
                                                       const SelectState *__restrict__ st,
                                                       int32_t *__restrict__ lo_out, int32_t *__restrict__ up_out)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= D) return;
    const float lv = __uint_as_float(st->reachable != 0 ? st->prefix : SEL_TOP);
    const float *ki = key + (size_t)i * MS;
    lo_out[i] = steps_below<false>(ki, MS, lv);
    up_out[i] = steps_below<true>(ki, MS, lv);
}

// Steps strictly below the level are all taken; those at the level in neuron order until the
// missing pairs are found; writes b = -tau, the pointers and the number of steps.  One block.
__global__ __launch_bounds__(SEL_THREADS) void k_select_finish(const int32_t *__restrict__ lo_in,
                                                               const int32_t *__restrict__ up_in,
                                                               const int32_t *__restrict__ drop,
                                                               const float *__restrict__ tauc,
                                                               const int32_t *__restrict__ k0, int D, int T, int eta,
                                                               int MS, const SelectState *__restrict__ st,
                                                               float *__restrict__ b, int32_t *__restrict__ k_out,
                                                               int32_t *__restrict__ steps)
{
    __shared__ long long red[SEL_THREADS / 64];
    __shared__ long long wave_tot[SEL_THREADS / 64];
    __shared__ int star;                                            // neuron at which the target is reached
    __shared__ long long star_before;                               // pairs found before its steps at the level
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool at_start = st->at_start != 0;
    const bool reachable = st->reachable != 0;
    const long long missing = st->missing;                          // among the steps at the level
    if (tid == 0) {
        star = D;
        star_before = 0;
    }
    __syncthreads();
    long long carried = 0;
    for (int i0 = 0; i0 < D && reachable; i0 += SEL_THREADS) {
        const int i = i0 + tid;
        long long gain = 0;
        if (i < D) {
            const int32_t *di = drop + (size_t)i * (MS + 1);
            gain = (long long)di[up_in[i]] - di[lo_in[i]];
        }
        long long inc = gain;                                       // inclusive scan inside the wave
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const long long o = __shfl_up(inc, off);
            if (lane >= off) inc += o;
        }
        if (lane == 63) wave_tot[wave] = inc;
        __syncthreads();
        long long before = carried;
        for (int q = 0; q < wave; ++q) before += wave_tot[q];
        long long chunk_total = 0;
        for (int q = 0; q < SEL_THREADS / 64; ++q) chunk_total += wave_tot[q];
        const long long excl = before + inc - gain;                 // found before this neuron's steps at the level
        if (i < D && excl < missing && excl + gain >= missing) {
            star = i;                                               // exactly one neuron satisfies this
            star_before = excl;
        }
        __syncthreads();
        carried += chunk_total;
        if (star < D) break;
    }
    __syncthreads();
    const int istar = star;
    const long long sb = star_before;
    long long taken = 0;
    for (int i = tid; i < D; i += SEL_THREADS) {
        const int32_t *di = drop + (size_t)i * (MS + 1);
        int J;
        if (at_start) {
            J = 0;
        } else if (!reachable || i < istar) {
            J = up_in[i];                                           // unreachable target: every finite step
        } else {
            J = lo_in[i];
            if (i == istar) {
                long long c = sb;
                while (c < missing) {                               // its steps at the level, one at a time
                    c += di[J + 1] - di[J];
                    ++J;
                }
            }
        }
        taken += J;
        b[i] = -tauc[(size_t)i * (MS + 1) + J];
        if (k_out != nullptr) k_out[i] = min(k0[i] + J * eta, T);
    }
    if (steps != nullptr) {
        const long long tot = block_sum_i64(taken, red);
        if (tid == 0) *steps = (int32_t)tot;
    }
}

}   // namespace svdp
