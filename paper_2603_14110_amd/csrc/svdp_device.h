// Device-side helpers for the gfx950 kernels: 16-byte weight loads widened to
// fp32, wave64 reductions on DPP, bf16 <-> fp32 bit conversions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace svdp {

// bfloat16 storage element (bit pattern only; all arithmetic is fp32, the
// "full precision registers, half precision memory" policy of the paper's App. C).
struct bf16 {
    uint16_t bits;
};

template <typename W>
struct Elem;
template <>
struct Elem<float> {
    static constexpr int VEC = 4;   // elements per 16-byte load
    static constexpr int BYTES = 4;
};
template <>
struct Elem<bf16> {
    static constexpr int VEC = 8;
    static constexpr int BYTES = 2;
};

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return __uint_as_float(((uint32_t)v.bits) << 16); }

// fp32 -> storage element, round-to-nearest-even (NaN stays NaN).
__device__ __forceinline__ void from_f32(float v, float *out) { *out = v; }
__device__ __forceinline__ void from_f32(float v, bf16 *out)
{
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) {
        out->bits = (uint16_t)((u >> 16) | 0x40u);
    } else {
        u += 0x7fffu + ((u >> 16) & 1u);
        out->bits = (uint16_t)(u >> 16);
    }
}

// One 16-byte load of VEC consecutive elements, widened to fp32.  p must be
// 16-byte aligned.
__device__ __forceinline__ void load_vec(const float *p, float (&v)[4])
{
    const float4 q = *reinterpret_cast<const float4 *>(p);
    v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
}
__device__ __forceinline__ void load_vec(const bf16 *p, float (&v)[8])
{
    const uint4 q = *reinterpret_cast<const uint4 *>(p);
    v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
    v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
    v[4] = __uint_as_float(q.z << 16); v[5] = __uint_as_float(q.z & 0xffff0000u);
    v[6] = __uint_as_float(q.w << 16); v[7] = __uint_as_float(q.w & 0xffff0000u);
}

// Raw 16-byte load (issued early, widened later) and its widening to fp32.
template <typename W>
__device__ __forceinline__ uint4 load_raw(const W *p)
{
    return *reinterpret_cast<const uint4 *>(p);
}
__device__ __forceinline__ void widen(const uint4 &q, float (&v)[4], const float *)
{
    v[0] = __uint_as_float(q.x); v[1] = __uint_as_float(q.y);
    v[2] = __uint_as_float(q.z); v[3] = __uint_as_float(q.w);
}
__device__ __forceinline__ void widen(const uint4 &q, float (&v)[8], const bf16 *)
{
    v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
    v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
    v[4] = __uint_as_float(q.z << 16); v[5] = __uint_as_float(q.z & 0xffff0000u);
    v[6] = __uint_as_float(q.w << 16); v[7] = __uint_as_float(q.w & 0xffff0000u);
}

// Dot product of two raw 16-byte vectors of storage elements, accumulated in fp32.
// bf16: four packed two-element dot instructions (bf16 x bf16 products are exact in
// fp32; the sum is rounded to fp32); fp32: four fused multiply-adds.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float dot_raw(const uint4 &w, const uint4 &x, float acc, const float *)
{
    acc = fmaf(__uint_as_float(w.x), __uint_as_float(x.x), acc);
    acc = fmaf(__uint_as_float(w.y), __uint_as_float(x.y), acc);
    acc = fmaf(__uint_as_float(w.z), __uint_as_float(x.z), acc);
    acc = fmaf(__uint_as_float(w.w), __uint_as_float(x.w), acc);
    return acc;
}
__device__ __forceinline__ float dot_raw(const uint4 &w, const uint4 &x, float acc, const bf16 *)
{
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.x), __builtin_bit_cast(bf16x2_t, x.x), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.y), __builtin_bit_cast(bf16x2_t, x.y), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.z), __builtin_bit_cast(bf16x2_t, x.z), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.w), __builtin_bit_cast(bf16x2_t, x.w), acc, false);
    return acc;
}

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

// Sum over the 64 lanes of a wave in a fixed order; the result is uniform.
// Four DPP steps give every lane the sum of its row of 16, then the four row
// sums are read out and added in lane order.
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);   // row_half_mirror
    v += dpp_move<0x140>(v);   // row_mirror
    const float a = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float b = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float c = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return (a + b) + (c + d);
}

// Inclusive prefix sum of one int per lane over the wave (lane order), on DPP row
// shifts and row broadcasts; lane 63 ends up with the wave total.
template <int CTRL, int ROW_MASK, int BANK_MASK>
__device__ __forceinline__ int dpp_take(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, BANK_MASK, true);
}
__device__ __forceinline__ int wave_inclusive_scan(int v)
{
    int s = v + dpp_take<0x111, 0xf, 0xf>(v);      // row_shr:1
    s += dpp_take<0x112, 0xf, 0xf>(v);             // row_shr:2
    s += dpp_take<0x113, 0xf, 0xf>(v);             // row_shr:3
    s += dpp_take<0x114, 0xf, 0xe>(s);             // row_shr:4, lanes 4..15 of each row
    s += dpp_take<0x118, 0xf, 0xc>(s);             // row_shr:8, lanes 8..15 of each row
    s += dpp_take<0x142, 0xa, 0xf>(s);             // row_bcast:15 into rows 1 and 3
    s += dpp_take<0x143, 0xc, 0xf>(s);             // row_bcast:31 into rows 2 and 3
    return s;
}

// Sum over aligned groups of 2^LOG2 consecutive lanes; every lane of a group
// gets the group's sum.  Butterfly order, fixed.
template <int LOG2>
__device__ __forceinline__ float group_sum(float v)
{
    if (LOG2 >= 1) v += dpp_move<0xB1>(v);
    if (LOG2 >= 2) v += dpp_move<0x4E>(v);
    if (LOG2 >= 3) v += dpp_move<0x141>(v);
    if (LOG2 >= 4) v += dpp_move<0x140>(v);
    if (LOG2 >= 5) v += __shfl_xor(v, 16);
    if (LOG2 >= 6) v += __shfl_xor(v, 32);
    return v;
}

}  // namespace svdp
