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
//   k_calib_sort   one block per neuron: bitonic sort of the samples by score in
//                  LDS (ties keep sample order), first positive weight, step
//                  costs (fp32, left to right), their running maxima, and for
//                  every step the number of dropped samples and the threshold
//                  it would set; optionally the Kendall check of App. A.
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
// Dynamic LDS: n2*8 (sort keys) + 2*T*4 (sorted s, w) + 2*(MS+1)*4 bytes, n2 = T rounded up to a power of two.
__global__ __launch_bounds__(CAL_THREADS) void k_calib_sort(const float *__restrict__ w, const float *__restrict__ s,
                                                            int T, int n2, int eta, int MS, float *__restrict__ key,
                                                            int32_t *__restrict__ drop, float *__restrict__ tauc,
                                                            int32_t *__restrict__ k0_out, float *__restrict__ kendall)
{
    extern __shared__ unsigned long long smem64[];
    unsigned long long *sk = smem64;                               // [n2]
    float *ss = reinterpret_cast<float *>(sk + n2);                // [T] sorted scores
    float *ww = ss + T;                                            // [T] weights in that order
    float *cost = ww + T;                                          // [MS + 1]
    float *scan = cost + (MS + 1);                                 // [MS + 1]
    __shared__ int first_pos;
    __shared__ int kd_total;
    const int i = blockIdx.x, tid = threadIdx.x;
    const float *si = s + (size_t)i * T, *wi = w + (size_t)i * T;

    for (int t = tid; t < n2; t += CAL_THREADS)
        sk[t] = t < T ? ((unsigned long long)ordered_bits(si[t]) << 32) | (unsigned)t : ~0ull;
    if (tid == 0) {
        first_pos = T;
        kd_total = 0;
    }
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
    for (int p = tid; p < T; p += CAL_THREADS) {
        const int t = (int)(sk[p] & 0xffffffffu);
        const float wv = wi[t];
        ss[p] = si[t];
        ww[p] = wv;
        if (wv > 0.f) atomicMin(&first_pos, p);
    }
    __syncthreads();
    const int k0 = first_pos < T ? first_pos + 1 : T;              // min{k : w_(k) > 0}, or T if there is none
    const int M = (T - k0 + eta - 1) / eta;                        // steps this neuron can take

    // step costs C(k + eta) - C(k), fp32 left to right; the last step may be short (the listing's padding)
    for (int j = tid; j < M; j += CAL_THREADS) {
        const int lo = k0 + j * eta, hi = min(lo + eta, T);
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
    // thresholds and dropped counts after j steps: k = min(k0 + j*eta, T), tau = s_(k), #{s <= tau}
    for (int j = tid; j <= MS; j += CAL_THREADS) {
        int dj = 0;
        float tj = 0.f;
        if (j <= M) {
            const int k = min(k0 + j * eta, T);
            tj = ss[k - 1];
            int lo = k, hi = T;                                     // first position whose score exceeds tau
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (ss[mid] <= tj) lo = mid + 1;
                else hi = mid;
            }
            dj = lo;
        }
        drop[(size_t)i * (MS + 1) + j] = dj;
        tauc[(size_t)i * (MS + 1) + j] = tj;
    }
    if (tid == 0) k0_out[i] = k0;

    if (kendall != nullptr) {
        // App. A: non-overlapping eta-step sums over the whole sorted sample, discordant pairs m1 < m2
        const int MK = T / eta;
        __syncthreads();                                            // cost/scan are free again
        float *S = cost;                                            // MK <= MS entries
        for (int m = tid; m < MK; m += CAL_THREADS) {
            float c = 0.f;
            for (int p = m * eta; p < (m + 1) * eta; ++p) c += ww[p];
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

// Picks the digit, updates the state and clears the histogram for the next digit.
template <int SHIFT, bool FIRST>
__global__ __launch_bounds__(64) void k_select_pick(SelectState *__restrict__ st, long long *__restrict__ hist)
{
    if (threadIdx.x != 0) return;
    if (st->reachable != 0) {
        long long run = 0;
        int digit = -1;
        const long long missing = st->missing;
        for (int q = 0; q < SEL_BINS; ++q) {
            if (digit < 0 && run + hist[q] >= missing) {
                digit = q;
                break;
            }
            run += hist[q];
        }
        if (digit < 0) {
            st->reachable = 0;                  // only on the first digit: every finite step together falls short
        } else {
            st->missing = missing - run;        // still to be found among the steps with this digit
            st->prefix |= (uint32_t)digit << SHIFT;
        }
    }
    for (int q = 0; q < SEL_BINS; ++q) hist[q] = 0;
}

// With the level known: steps strictly below it are all taken; those at the level in neuron order
// until the missing pairs are found; writes b = -tau, the pointers and the number of steps.
__global__ __launch_bounds__(SEL_THREADS) void k_select_finish(const float *__restrict__ key,
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
    const float lv = __uint_as_float(reachable ? st->prefix : SEL_TOP);
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
            const float *ki = key + (size_t)i * MS;
            const int32_t *di = drop + (size_t)i * (MS + 1);
            gain = (long long)di[steps_below<true>(ki, MS, lv)] - di[steps_below<false>(ki, MS, lv)];
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
        const float *ki = key + (size_t)i * MS;
        const int32_t *di = drop + (size_t)i * (MS + 1);
        int J;
        if (at_start) {
            J = 0;
        } else if (!reachable) {
            J = steps_below<true>(ki, MS, lv);                      // every finite step: the target cannot be met
        } else if (i < istar) {
            J = steps_below<true>(ki, MS, lv);
        } else {
            J = steps_below<false>(ki, MS, lv);
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
