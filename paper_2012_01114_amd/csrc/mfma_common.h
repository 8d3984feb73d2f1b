// Vector types and small helpers for the gfx950 MFMA kernels.
#pragma once

#include "common.h"

namespace attnring {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// v_mfma_f32_32x32x16_bf16: D[32x32] += A[32x16] * B[16x32], one wavefront.
// Lane L supplies row (L % 32) of A and column (L % 32) of B, eight consecutive
// k each, starting at k = 8 * (L / 32).  Lane L receives column (L % 32) of D;
// its register r holds row 8 * (r / 4) + 4 * (L / 32) + (r % 4).
__device__ __forceinline__ f32x16 mfma32(u32x4 a, u32x4 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                   0, 0, 0);
}

// v_mfma_f32_32x32x16_f16: the same shape and lane layout on half-precision operands, the type
// of the projected q, k, v and of the exponentials between the two kernels of a forward pass.
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ f32x16 mfma32h(u32x4 a, u32x4 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c,
                                                  0, 0, 0);
}

// Row (within a 32-row block) held by accumulator register r of a lane in half g.
__device__ __forceinline__ constexpr int acc_row(int r, int g) { return 8 * (r >> 2) + 4 * g + (r & 3); }

// Two floats -> two bfloat16 (round to nearest even) packed in one dword.
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}

// Two floats -> two half-precision values (round to nearest even) packed in one dword.
__device__ __forceinline__ unsigned pack_f16(float lo, float hi)
{
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, f16x2));
}
// The same for projected q, k, v: values beyond the half-precision range saturate at its
// largest finite value instead of becoming infinite.
__device__ __forceinline__ unsigned pack_f16_sat(float lo, float hi)
{
    constexpr float HMAX = 65504.f;
    return pack_f16(__builtin_amdgcn_fmed3f(lo, -HMAX, HMAX), __builtin_amdgcn_fmed3f(hi, -HMAX, HMAX));
}

// Position of key (j % 16) inside its 16-key group of the transposed V layout:
// bits 2 and 3 exchanged, so that the eight keys a lane half owns in the
// accumulator layout (acc_row) are contiguous.
__device__ __host__ __forceinline__ constexpr int vt_slot16(int r16)
{
    return (r16 & 3) | ((r16 & 4) << 1) | ((r16 & 8) >> 1);
}

}  // namespace attnring
