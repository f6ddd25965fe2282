// The per-token, per-64-group int4 quantiser chain (eq. 5, 8, 9, 3) on the 32 values a lane holds of one group:
// shared by the quantise kernel and by the GEMM epilogue that emits the next layer's operands itself.
#pragma once
#include "svdq_dev.h"

namespace svdq {

// max over the two lanes (l, l^32) that share a token row.  The compiler builtin
// (not inline asm) so that the wait states v_permlane32_swap needs after a VALU
// write of its operands are inserted.
__device__ __forceinline__ float max_pair32(float v) {
    const uint32_t a = f_bits(v);
    auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
    return fmaxf(bits_f(r[0]), bits_f(r[1]));
}

// s = t / 7 with one multiply and two FMAs.  With y = RN(1/7): q0 = RN(t*y), r = t - 7*q0 (exact in
// an FMA), q1 = RN(q0 + r*y).  Checked exhaustively on the host against IEEE division for every
// binary32 mantissa; tiny t (results near the denormal range) take the IEEE sequence.
__device__ __forceinline__ float div7(float t) {
    const float y7 = 0.142857149243354797363281250f;
    float q0 = __fmul_rn(t, y7);
    float rem = __builtin_fmaf(-7.0f, q0, t);
    float q1 = __builtin_fmaf(rem, y7, q0);
    return (t >= 7.8886090522101181e-31f) ? q1 : __fdiv_rn(t, 7.0f);          // 2^-100
}

// RN(1/s) from v_rcp_f32 (1 ulp) and one FMA Newton step.  Equal to IEEE division for every mantissa
// on gfx950 as long as 1/s is a normal number (the GPU tests sweep every mantissa through
// scale_chain_kernel below); huge s takes the IEEE sequence.
__device__ __forceinline__ float recip_rn(float s) {
    float r0 = __builtin_amdgcn_rcpf(s);
    float e = __builtin_fmaf(-s, r0, 1.0f);
    float r1 = __builtin_fmaf(e, r0, r0);
    return (s <= 4.2535295865117308e+37f) ? r1 : __fdiv_rn(1.0f, s);           // 2^125
}

constexpr uint32_t RNE_MAGIC_BITS = 0x4B400008u;            // 1.5*2^23 + 8: rounds to integer, biases codes to [0,15]
// sum_i RNE_MAGIC_BITS-without-the-8 * 16^i mod 2^32: what the magic's exponent bits add up to when eight
// results are folded with w = (w << 4) + t
constexpr uint32_t PACK_JUNK = (uint32_t)(0x4B400000ull * 0x11111111ull);

// Codes of one lane: 32 consecutive k of one token row.  Nibbles: 16 bytes, two's complement, k ascending from
// the low nibble of byte 0.  E3M2: the same integers as 6-bit floating-point fields (sign, 3 exponent bits of
// bias 3, 2 mantissa bits; every integer in [-8, 8] is exact there), 24 bytes, k ascending from bit 0: the
// operand format of the FP6 matrix instructions, which run at twice the int8 rate.
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x6 __attribute__((ext_vector_type(6)));
template <bool E3M2> struct LaneCodes { uint4 lo; uint2 hi; };

// One 32-row block of one group: quantiser chain on this lane's 32 values.
template <bool E3M2>
__device__ __forceinline__ void quantize_rows(const uint4 (&xv)[4], const float* __restrict__ il_lds, float rho,
                                              LaneCodes<E3M2>& codes, float& s_out) {
    float xs[32];
    float a = 0.0f;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const float4 i0 = *reinterpret_cast<const float4*>(il_lds + 8 * s);
        const float4 i1 = *reinterpret_cast<const float4*>(il_lds + 8 * s + 4);
        const float ilv[8] = {i0.x, i0.y, i0.z, i0.w, i1.x, i1.y, i1.z, i1.w};
        const uint32_t wds[4] = {xv[s].x, xv[s].y, xv[s].z, xv[s].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float lo = __fmul_rn(bf16lo_f(wds[j]), ilv[2 * j]);          // eq. 5 in binary32
            float hi = __fmul_rn(bf16hi_f(wds[j]), ilv[2 * j + 1]);
            xs[8 * s + 2 * j] = lo;
            xs[8 * s + 2 * j + 1] = hi;
            a = __builtin_fmaxf(a, __builtin_fmaxf(__builtin_fabsf(lo), __builtin_fabsf(hi)));
        }
    }
    a = max_pair32(a);                                                  // reference magnitude of eq. 8

    // eq. 8-9: s = (rho * a) / q_max ; zero or denormal scale -> empty group
    float s = div7(__fmul_rn(rho, a));
    const bool live = s >= 1.17549435e-38f;
    s = live ? s : 0.0f;
    const float inv = live ? recip_rn(s) : 0.0f;
    s_out = s;

    // eq. 3: clip(rne(x^ * (1/s)), -8, 7).  Clamping before rounding gives the same code.  Adding
    // 1.5*2^23 + 8 rounds to nearest-even and leaves code + 8 (0..15) in the low mantissa bits, so eight
    // results fold into a dword with shift-adds and no carries between nibbles; the folded exponent
    // bits are a constant, and x ^ 8 turns a biased nibble back into two's complement.
    if constexpr (E3M2) {
        // same decision (clamp, then round to nearest even integer), then the hardware conversion of the 32
        // integer-valued floats to E3M2 fields, which is exact on them.  It interleaves its two inputs:
        // field 2 j comes from the first vector, field 2 j + 1 from the second.
        f32x16 ev, od;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const float u0 = __builtin_amdgcn_fmed3f(__fmul_rn(xs[2 * j], inv), -8.0f, 7.0f);
            const float u1 = __builtin_amdgcn_fmed3f(__fmul_rn(xs[2 * j + 1], inv), -8.0f, 7.0f);
            ev[j] = __builtin_rintf(u0);
            od[j] = __builtin_rintf(u1);
        }
        const u32x6 c = __builtin_amdgcn_cvt_scalef32_2xpk16_bf6_f32(ev, od, 1.0f);
        codes.lo = uint4{c[0], c[1], c[2], c[3]};
        codes.hi = uint2{c[4], c[5]};
        return;
    }
    uint32_t packed[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        uint32_t wd = 0;
#pragma unroll
        for (int j = 7; j >= 0; --j) {
            float u = __fmul_rn(xs[8 * d + j], inv);
            u = __builtin_amdgcn_fmed3f(u, -8.0f, 7.0f);
            uint32_t t = f_bits(__fadd_rn(u, bits_f(RNE_MAGIC_BITS)));
            wd = (wd << 4) + t;
        }
        packed[d] = (wd - PACK_JUNK) ^ 0x88888888u;
    }
    codes.lo = uint4{packed[0], packed[1], packed[2], packed[3]};
}

}  // namespace svdq
