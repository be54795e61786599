// Shared device-side types and small helpers for the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define RS_DEVICE static __device__ __forceinline__

constexpr int WAVE = 64;

RS_DEVICE float bf16_to_f32(bf16 v) { return (float)v; }
RS_DEVICE bf16 f32_to_bf16(float v) { return (bf16)v; }   // round-to-nearest-even (v_cvt_pk_bf16_f32)

RS_DEVICE float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, WAVE);
    return v;
}

// 16-byte global / LDS accessors on raw byte pointers.
RS_DEVICE uint4 ld_global_16(const void* p) { return *reinterpret_cast<const uint4*>(p); }
RS_DEVICE void st_global_16(void* p, uint4 v) { *reinterpret_cast<uint4*>(p) = v; }

RS_DEVICE bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }
RS_DEVICE uint4 as_uint4(bf16x8 v) { return __builtin_bit_cast(uint4, v); }
