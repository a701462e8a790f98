// Vector types, constants and small device helpers shared by the matrix-core decode kernels.
#pragma once
#include "mla_internal.h"

namespace mla {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

#define LDS_AS __attribute__((address_space(3)))
#define CONST_AS __attribute__((address_space(4)))

constexpr int MF_THREADS = 256;
constexpr int TILE_ROWS = 32;     // cached rows per tile (half a page)
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float RESCALE_GAP = 32.f;   // careful pass: move the reference when exceeded by this
constexpr float FAST_GAP = 64.f;      // fast pass: largest excess over the fixed reference it tolerates

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// two fp32 -> packed bf16x2, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){lo, hi}, bf16x2));
}

// chunk swizzle key of tile row r: bits (r2, r1, r3).  Rows r and r+2 differ in bit 1 of the
// key (different 32-byte block), rows r and r+4 in bit 2, rows r and r+8 in bit 0.
__device__ __forceinline__ constexpr int swz_key(int r)
{
    return (((r >> 2) & 1) << 2) | (((r >> 1) & 1) << 1) | ((r >> 3) & 1);
}

// s_waitcnt vmcnt(N) with the other counters left alone (gfx9 encoding)
template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

}  // namespace mla
