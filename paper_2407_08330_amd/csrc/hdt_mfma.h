// Small device helpers shared by the bf16 MFMA kernels (gfx950 / CDNA4, wave64).
//
// Register layouts of v_mfma_f32_32x32x16_bf16 (checked on the hardware with one-hot inputs):
//   A (32 x 16) : lane l holds row  l%32, k = (l/32)*8 + 0..7   (8 bf16 = 4 VGPRs)
//   B (16 x 32) : lane l holds col  l%32, k = (l/32)*8 + 0..7
//   C (32 x 32) : lane l holds col  l%32, rows (l/32)*4 + 8*(v/4) + v%4 for v = 0..15
// The contraction index only has to be labelled the same way in A and B, so a C fragment
// can be fed back as a B operand without moving data between lanes: registers v = 8*ks .. 8*ks+7
// of lane (col, hf) hold rows {16*ks + hf*4 + 0..3} and {16*ks + 8 + hf*4 + 0..3}, and the A operand
// of that step is loaded for exactly those 8 contraction indices.
//
// ds_read_b64_tr_b16 (checked the same way): inside each group of 16 lanes, lane t supplies the
// address of 4 consecutive b16 values; the group's 16 x 4 values form 4 rows of 16 (row j = lanes
// 4j..4j+3), and lane t receives element t of rows 0..3.  Reading a row-major [k][n] tile this way
// gives every lane 4 consecutive k at one n: the operand layout the MFMA wants for a matrix
// whose contraction index is the slow one in memory.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

#define HDT_LDS __attribute__((address_space(3)))

__device__ __forceinline__ f32x16 mfma_32x32x16(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// 8 bf16 from 16 contiguous bytes of LDS
__device__ __forceinline__ bf16x8 lds_read_8(const char *p)
{
    return *reinterpret_cast<const bf16x8 *>(p);
}

// two transposing reads -> the 8 contraction values of one MFMA operand
__device__ __forceinline__ bf16x8 lds_read_tr_8(const char *p0, const char *p1)
{
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((HDT_LDS s16x4 *)(p0));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((HDT_LDS s16x4 *)(p1));
    s16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

__device__ __forceinline__ bf16x8 zero_bf16x8()
{
    const s16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    return __builtin_bit_cast(bf16x8, z);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ bf16x8 pack_bf16x8(const f32x16 &p, int first)
{
    bf16x8 r;
#pragma unroll
    for (int i = 0; i < 8; i++) r[i] = (__bf16)p[first + i];
    return r;
}
