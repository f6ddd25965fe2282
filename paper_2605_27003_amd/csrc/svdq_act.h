// Activation fused into the quantise pass: GELU in its tanh form, as the feed-forward block of the DiT applies it
// between the up- and the down-projection, evaluated on the bf16 value and rounded back to bf16 (what a separate
// element-wise kernel would have written), so that the quantise kernel of the down-projection can take the
// up-projection's output directly and one write and one read of that tensor disappear.
#pragma once
#include "svdq_dev.h"

namespace svdq {

// gelu(x) = x / (1 + exp(-z)), z = 2 sqrt(2/pi) (x + 0.044715 x^3)   [ = 0.5 x (1 + tanh(z / 2)) ], for a bf16 x,
// to be rounded to bf16 by the caller.  The function has only 65 536 inputs, so it is DEFINED by its table: the
// CPU reference evaluates a fixed, correctly rounded binary32 sequence (polynomial exp, IEEE division), and this
// code uses the hardware's exp2 and reciprocal approximations (7 instead of ~40 vector instructions), whose
// errors of about one binary32 ulp never reach a bf16 rounding boundary: the GPU test compares the two on every
// finite bf16 input.  Beyond -z > 87 the reference returns 0 (its exp would overflow); the select below does the
// same.  Finite inputs.
__device__ __forceinline__ float gelu_tanh_f32(float x) {
    const float u = __fmul_rn(x, x);
    const float p = __builtin_fmaf(0.044715f, u, 1.0f);
    const float t = __fmul_rn(x, p);
    const float z = __fmul_rn(1.5957691216057308f, t);
    const float e = __builtin_amdgcn_exp2f(__fmul_rn(t, -1.5957691216057308f * 1.44269504088896341f));   // exp(-z)
    float sig = __builtin_amdgcn_rcpf(__fadd_rn(1.0f, e));
    sig = (-z > 87.0f) ? 0.0f : sig;
    return __fmul_rn(x, sig);
}

// two bf16 values in a dword -> gelu of both, rounded to bf16 (nearest even)
__device__ __forceinline__ uint32_t gelu_tanh_bf16x2(uint32_t w) {
    return f2_bf16_rne(gelu_tanh_f32(bf16lo_f(w)), gelu_tanh_f32(bf16hi_f(w)));
}

// the 32 values a lane holds of one 64-group
__device__ __forceinline__ void gelu_tanh_rows(uint4 (&xv)[4]) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        xv[s].x = gelu_tanh_bf16x2(xv[s].x);
        xv[s].y = gelu_tanh_bf16x2(xv[s].y);
        xv[s].z = gelu_tanh_bf16x2(xv[s].z);
        xv[s].w = gelu_tanh_bf16x2(xv[s].w);
    }
}

}  // namespace svdq
