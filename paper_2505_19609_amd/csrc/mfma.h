// CDNA4 (gfx950) device helpers shared by the attention kernels: vector types,
// the 32x32x16 bf16 MFMA, LDS swizzles, packed conversions.
//
// MFMA v_mfma_f32_32x32x16_bf16 computes D[32x32] += A[32x16] * B[16x32] per
// 64-lane wavefront.  Lane l = 32*h + n (h = 0/1, n = 0..31) supplies
//   A: row n,    eight consecutive k:  A[n][8h .. 8h+7]
//   B: column n, eight consecutive k:  B[8h .. 8h+7][n]
// and holds, in accumulator register v = 0..15,
//   D[8*(v/4) + 4*h + (v%4)][n].
// So a lane owns ONE column of the result and 16 of its rows.  The kernels put
// the query index on the column wherever a per-query scalar (running max,
// row sum, LSE, D) multiplies the tile, which keeps those scalars lane-local.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 u) { return __builtin_bit_cast(bf16x8, u); }

// Two floats -> packed bf16 pair (round to nearest even), one v_cvt_pk_bf16_f32.
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    f32x2 f = {lo, hi};
    bf16x2 b = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

