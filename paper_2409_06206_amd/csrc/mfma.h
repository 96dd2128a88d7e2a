// MFMA building blocks for the fused GSWA kernels (gfx950, wave64).
//
// Fragment conventions used everywhere in the fused kernels, for the 16x16xK bf16 MFMAs
// D[16x16] += A[16xK] * B[Kx16], with l16 = lane & 15 and q = lane >> 4:
//   A operand: the lane holds row l16, k-slots q*KV .. q*KV + KV-1   (KV = 4 for K=16, 8 for K=32)
//   B operand: the lane holds column l16, the same k-slots
//   D result : the lane holds column l16, rows 4q .. 4q+3            ("C layout")
// Two consequences the kernels are built on:
//   * a C-layout tile X (rows i, columns j), packed to bf16, IS the B operand "X" and the A
//     operand "X^T" of a K=16 MFMA that reduces over X's row index i;
//   * swapping the two operands of an MFMA yields the transposed product, so either
//     orientation of a result costs no data movement.
// The k-slot order only has to agree between the two operands, so any consistent permutation
// of the reduction index is allowed (used to chain padded head tiles).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gswa {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// two fp32 -> two bf16 (round to nearest even), low half = a
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
    f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ __forceinline__ uint2 pack_bf16x4(f32x4 v)
{
    return make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
}

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// D += A * B, K = 16: operands hold 4 bf16 per lane
__device__ __forceinline__ f32x4 mma16(uint2 a, uint2 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, a),
                                                     __builtin_bit_cast(s16x4, b), c, 0, 0, 0);
}

// D += A * B, K = 32: operands hold 8 bf16 per lane
__device__ __forceinline__ f32x4 mma32(uint4 a, uint4 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// all-reduce over the four lanes that share l16 (q = 0..3), without touching LDS:
// v_permlane16_swap(v, v) returns {rows 0,0,2,2 of v; rows 1,1,3,3 of v} (rows = 16 lanes), and
// v_permlane32_swap(w, w) returns {lower half twice; upper half twice}.
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float qgroup_max(float v)
{
    const unsigned u = __float_as_uint(v);
    u32x2 r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const unsigned w = __float_as_uint(fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1])));
    r = __builtin_amdgcn_permlane32_swap(w, w, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float qgroup_sum(float v)
{
    const unsigned u = __float_as_uint(v);
    u32x2 r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const unsigned w = __float_as_uint(__uint_as_float(r[0]) + __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane32_swap(w, w, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Global memory as a buffer resource: uniform base + 32-bit byte offset per lane (+ a uniform
// offset and an immediate), so that no access needs a 64-bit address register; reads past
// `bytes` return zero and writes there are dropped.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __amdgpu_buffer_rsrc_t buf_t;
__device__ __forceinline__ buf_t make_buf(const void *p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ uint2 bload64(buf_t b, uint32_t voff, uint32_t soff)
{
    const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(b, (int)voff, (int)soff, 0);
    return make_uint2(v[0], v[1]);
}
__device__ __forceinline__ void bstore32(buf_t b, uint32_t voff, uint32_t soff, uint32_t v)
{
    __builtin_amdgcn_raw_buffer_store_b32(v, b, (int)voff, (int)soff, 0);
}
__device__ __forceinline__ void bstore64(buf_t b, uint32_t voff, uint32_t soff, uint2 v)
{
    const u32x2 w = {v.x, v.y};
    __builtin_amdgcn_raw_buffer_store_b64(w, b, (int)voff, (int)soff, 0);
}

} // namespace gswa
