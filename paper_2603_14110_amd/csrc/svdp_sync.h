// Hand-over of results between the blocks of ONE launch through global memory:
// producers write their results through to memory (agent-scope stores), wait
// until the writes are acknowledged and bump a counter; consumers poll the
// counters (bounded) and read the results with agent-scope loads.  Used where a
// kernel boundary would cost more than the wait.  Needs every block of the
// launch resident at once.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace svdp {

constexpr int CTRL_GROUPS = 8;          // counters per stage (arrivals are spread over them)
constexpr int CTRL_STRIDE = 32;         // 32-bit words between counters: one 128-byte line each
constexpr int CTRL_T = 0;               // word offsets of the three counter groups
constexpr int CTRL_M = CTRL_GROUPS * CTRL_STRIDE;
constexpr int CTRL_Y = 2 * CTRL_GROUPS * CTRL_STRIDE;
constexpr int CTRL_EXIT = 3 * CTRL_GROUPS * CTRL_STRIDE;
constexpr int CTRL_ERROR = CTRL_EXIT + CTRL_STRIDE;
constexpr int CTRL_WORDS = CTRL_ERROR + CTRL_STRIDE;     // 832 words per control block
constexpr int CTRL_SLOTS = 64;          // control blocks (one per workspace in use)

// ---- agent-scope accesses: visible across the chip's L2 caches without a cache flush ----
__device__ __forceinline__ void store_wt(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_wt(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float4 load_wt4(const float *p)
{
    return make_float4(load_wt(p), load_wt(p + 1), load_wt(p + 2), load_wt(p + 3));
}
// 16-byte forms of the two accesses above (one instruction instead of four).
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_wt16(float *p, float a, float b, float c, float d)
{
    const f32x4_t v = {a, b, c, d};
    // the trailing wait states cover the hazard between a 16-byte store and a following
    // write of its data registers, which the compiler cannot see through inline assembly
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 2" : : "v"(p), "v"(v) : "memory");
}
// four independent 16-byte loads in flight together; returns after all have arrived
__device__ __forceinline__ void load_wt16x4(const float *p0, const float *p1, const float *p2, const float *p3,
                                            f32x4_t &a, f32x4_t &b, f32x4_t &c, f32x4_t &d)
{
    asm volatile(
        "global_load_dwordx4 %0, %4, off sc1\n\t"
        "global_load_dwordx4 %1, %5, off sc1\n\t"
        "global_load_dwordx4 %2, %6, off sc1\n\t"
        "global_load_dwordx4 %3, %7, off sc1\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(a), "=&v"(b), "=&v"(c), "=&v"(d)
        : "v"(p0), "v"(p1), "v"(p2), "v"(p3)
        : "memory");
}
// all of this wave's outstanding global stores have been acknowledged
__device__ __forceinline__ void wait_stores_done() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0)

__device__ __forceinline__ void signal(uint32_t *ctrl, int group_base, int member)
{
    __hip_atomic_fetch_add(ctrl + group_base + (member % CTRL_GROUPS) * CTRL_STRIDE, 1u, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
}
// how many of `total` members (0..total-1) signal counter c
__device__ __forceinline__ uint32_t members_of(int total, int c) { return (uint32_t)((total - c + CTRL_GROUPS - 1) / CTRL_GROUPS); }

// Wave 0 polls the CTRL_GROUPS counters of one stage until each has seen all its
// members; bounded.  Call from every thread of the block.
__device__ __forceinline__ void wait_stage(uint32_t *ctrl, int group_base, int total, int spin_limit)
{
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        bool done = lane >= CTRL_GROUPS;
        const uint32_t target = done ? 0u : members_of(total, lane);
        int spins = 0;
        while (__ballot(!done) != 0ull) {
            if (!done)
                done = __hip_atomic_load(ctrl + group_base + lane * CTRL_STRIDE, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT) >= target;
            if (++spins > spin_limit) {
                if (lane == 0) __hip_atomic_store(ctrl + CTRL_ERROR, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
    }
    __syncthreads();
}

}  // namespace svdp
