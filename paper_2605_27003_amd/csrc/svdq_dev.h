// Device-side helpers shared by the gfx950 kernels of the W4A4 SVDQuant-style
// linear layer.  CDNA4 only: 64-wide wavefronts, MFMA matrix cores.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace svdq {

typedef int   int4v   __attribute__((ext_vector_type(4)));
typedef int   int16v  __attribute__((ext_vector_type(16)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));

constexpr int GROUP = 64;            // quantisation group along K
constexpr float QMAX = 7.0f;         // q_max of the int4 grid; codes are clamped to [-8, 7]

__device__ __forceinline__ float bits_f(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t f_bits(float f) { return __float_as_uint(f); }

// bf16 pair packed in a dword -> two binary32 values (exact widening).
__device__ __forceinline__ float bf16lo_f(uint32_t w) { return bits_f(w << 16); }
__device__ __forceinline__ float bf16hi_f(uint32_t w) { return bits_f(w & 0xffff0000u); }

// binary32 -> bf16 bits, round-to-nearest-even: the hardware conversion (v_cvt_pk_bf16_f32, two values per
// instruction).  On every finite input it returns what the integer sequence u += 0x7fff + ((u >> 16) & 1), u >> 16
// returns (all 2^32 patterns compared on the device), denormals and the overflow to infinity included.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float float2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f2_bf16_rne(float lo, float hi) {            // lo -> bits 0..15, hi -> bits 16..31
    const float2v v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ uint32_t f_bf16_rne(float f) { return f2_bf16_rne(f, 0.0f); }

}  // namespace svdq
