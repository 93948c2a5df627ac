// MFMA fragment helpers for gfx950 (wave64).
//
// Both operand fragments of the 32x32 MFMA shapes used here have the same lane layout:
// lane l supplies 16 bytes of row (l % 32) taken at K-byte offset chunk*32 + (l / 32)*16.
// The contraction only requires that both operands use the same lane -> K mapping, so a
// 16-byte piece is fed as one 32x32x16 f16 MFMA (8 halves) or as four 32x32x2 f32 MFMAs.
// Output (16 accumulators per lane): accumulator r of lane l is element
//   row = 8*(r/4) + 4*(l/32) + (r%4)   of the first operand's rows,
//   col = l % 32                       of the second operand's rows.
#pragma once
#include <hip/hip_runtime.h>

typedef _Float16 tri_half8 __attribute__((ext_vector_type(8)));
typedef float tri_f32x16 __attribute__((ext_vector_type(16)));

enum { TRI_DT_F32 = 0, TRI_DT_F16 = 1 };

template <int DT>
__device__ __forceinline__ void tri_mma32(tri_f32x16 &acc, const uint4 &a, const uint4 &b);

template <>
__device__ __forceinline__ void tri_mma32<TRI_DT_F16>(tri_f32x16 &acc, const uint4 &a, const uint4 &b)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(tri_half8, a), __builtin_bit_cast(tri_half8, b),
                                                 acc, 0, 0, 0);
}

template <>
__device__ __forceinline__ void tri_mma32<TRI_DT_F32>(tri_f32x16 &acc, const uint4 &a, const uint4 &b)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
}
