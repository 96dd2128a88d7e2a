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

#include <type_traits>
#include <utility>

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
__device__ __forceinline__ uint4 bload128(buf_t b, uint32_t voff, uint32_t soff)
{
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(b, (int)voff, (int)soff, 0);
    return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void bstore128(buf_t b, uint32_t voff, uint32_t soff, uint4 v)
{
    const u32x4 w = {v.x, v.y, v.z, v.w};
    __builtin_amdgcn_raw_buffer_store_b128(w, b, (int)voff, (int)soff, 0);
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

// One load instruction that writes LDS directly: lane l's 16 bytes at `src` (a per-lane address) land at
// the wave-uniform LDS address `dst` + 16 l.  Asynchronous: the data is in LDS once the wave's
// vector-memory counter has drained (s_waitcnt vmcnt(0)), which the caller does before the barrier
// that hands the data to its readers; the compiler is not told that LDS changes, so it adds no wait
// of its own to later LDS reads (they must not touch the destination before that barrier).  M0 is
// written here; the compiler reserves it and sets it itself before each of its own uses.
__device__ __forceinline__ void lds_dma16(const void *src, void *dst)
{
    const uint32_t ldsaddr =
        __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)dst);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(ldsaddr), "v"(src) : "memory");
}

__device__ __forceinline__ uint4 cat(uint2 a, uint2 b) { return make_uint4(a.x, a.y, b.x, b.y); }

// Two packed result tiles that are neighbours along their rows (lane group q of `a` holds rows 4q..4q+3
// of a 16-row run, of `b` the same rows of the next run) -> lane group q holds rows 8q..8q+7 of the
// 32-row run [a | b]: 16 contiguous bytes per lane, so that a column leaves in two stores of 32 bytes
// per lane pair instead of four of 8.  v_permlane32_swap(d, s): d' = {d.lower half, s.lower half},
// s' = {d.upper, s.upper}; v_permlane16_swap(d, s): d' = rows (d0, s0, d2, s2), s' = rows (d1, s1, d3, s3).
__device__ __forceinline__ uint4 pair_rows(uint2 a, uint2 b)
{
    const u32x2 r0 = __builtin_amdgcn_permlane32_swap(a.x, b.x, false, false);
    const u32x2 r1 = __builtin_amdgcn_permlane32_swap(a.y, b.y, false, false);
    const u32x2 s0 = __builtin_amdgcn_permlane16_swap(r0[0], r0[1], false, false);
    const u32x2 s1 = __builtin_amdgcn_permlane16_swap(r1[0], r1[1], false, false);
    return make_uint4(s0[0], s1[0], s0[1], s1[1]);
}

// Transposed store of a packed result tile (this lane: rows 4q..4q+3 of column l16) into
// row-major LDS rows.  Neighbouring lanes l16, l16^1 swap halves through DPP so that every lane
// writes whole dwords: even lanes rows 4q and 4q+2, odd lanes rows 4q+1 and 4q+3, each holding
// the columns (l16 & ~1, l16 | 1).  `row0` points at row 4q, column l16 & ~1.
__device__ __forceinline__ void store_tile_transposed(uint16_t *row0, int pitch, uint2 tile, int lane)
{
    const int odd = lane & 1;
    const uint32_t px = (uint32_t)__builtin_amdgcn_mov_dpp((int)tile.x, 0xB1, 0xF, 0xF, true); // quad_perm [1,0,3,2]
    const uint32_t py = (uint32_t)__builtin_amdgcn_mov_dpp((int)tile.y, 0xB1, 0xF, 0xF, true);
    const uint32_t sel = odd ? 0x03020706u : 0x05040100u;
    // even: lo16(own) | lo16(partner) << 16 ;  odd: hi16(partner) | hi16(own) << 16
    const uint32_t vx = __builtin_amdgcn_perm(px, tile.x, sel); // selector bytes 4-7 pick from px, 0-3 from own
    const uint32_t vy = __builtin_amdgcn_perm(py, tile.y, sel);
    uint32_t *d = reinterpret_cast<uint32_t *>(row0 + odd * pitch);
    d[0] = vx;
    d[pitch] = vy; // two rows further: 2 * pitch halves = pitch dwords
}

// K=32 operand that is 1.0 in the k-slot holding index `target` and 0 elsewhere, for a lane
// whose slots 0..7 hold indices first .. first+7.  Multiplying by it moves a matrix held as an
// operand (k-slots = columns) into result layout exactly: a transposition done by the MFMA unit.
__device__ __forceinline__ uint4 select_slot(int target, int first)
{
    const int sl = target - first;
    const uint32_t one = (sl & 1) ? 0x3f800000u : 0x00003f80u;
    const int dw = (sl >= 0 && sl < 8) ? (sl >> 1) : -1;
    return make_uint4(dw == 0 ? one : 0u, dw == 1 ? one : 0u, dw == 2 ? one : 0u, dw == 3 ? one : 0u);
}


// packed bf16 pairs, added in fp32 and rounded once
__device__ __forceinline__ uint32_t add_bf16x2(uint32_t a, uint32_t b)
{
    return pack_bf16x2(bf16_lo(a) + bf16_lo(b), bf16_hi(a) + bf16_hi(b));
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop whose index is a constant
// expression inside the body (register arrays indexed by it never need memory).
template <class F, int... I> __device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F> __device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(static_cast<F &&>(f), std::make_integer_sequence<int, N>{});
}

} // namespace gswa
