// Low-rank up-projection and bias of eq. 7 / eq. 11 on a wave's accumulator tile, shared by the GEMM kernels.
#pragma once
#include "svdq_dev.h"

namespace svdq {

// y[ni][mi] += (h L2)^T + bias for a wave tile of NI 32-channel blocks (first channel n0) times MT 32-token
// blocks (first token m0), in the accumulator layout of the 32x32 matrix instructions with the transposed
// tile D[n][m]: lane (l32 = lane % 32, kh = lane / 32) owns token m0 + 32 mi + l32 and, in register i,
// channel n0 + 32 ni + 8 (i / 4) + 4 kh + (i % 4).
//
// h [M, r] binary32 is split into hi + lo bf16 pieces and multiplied by the bf16 L2 [r, N] on the bf16 matrix
// cores (v_mfma_f32_32x32x16_bf16, L2^T as the A operand), two instructions per 16 of r.  r is 0, 16 or 32.
// ALL global loads are issued before the first use: the code path is the same for r = 16 and r = 32 (the second
// k-step then reads valid addresses and its L2 fragment is zeroed), so their latency is paid once, not per
// k-step.  Rows beyond M are clamped for the loads (their results are never stored).
//
// h_piece(mi, k) returns the four values h[token of block mi][k .. k + 3] of this lane's token (k a multiple of 4):
// from global memory in add_lowrank_bias, from wherever the caller staged the tile's h rows in add_lowrank_bias_from.
template <int NI, int MT, class HPiece>
__device__ __forceinline__ void add_lowrank_bias_from(float16v (&y)[NI][MT], HPiece h_piece,
                                                      const uint16_t* __restrict__ L2, const float* __restrict__ bias,
                                                      int n0, int N, int r, int lane) {
    const int l32 = lane & 31, kh = lane >> 5;
    float4 bv[NI][4];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            bv[ni][q] = float4{0.f, 0.f, 0.f, 0.f};
            if (bias) bv[ni][q] = *reinterpret_cast<const float4*>(bias + n0 + ni * 32 + 8 * q + 4 * kh);
        }
    if (r > 0) {
        uint32_t wds[2][NI][4];
        float4 hv[2][MT][2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int k0 = (16 * ks < r) ? 16 * ks : 0;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const int n = n0 + ni * 32 + l32;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t lo = L2[(int64_t)(k0 + 8 * kh + 2 * e) * N + n];
                    const uint32_t hi = L2[(int64_t)(k0 + 8 * kh + 2 * e + 1) * N + n];
                    wds[ks][ni][e] = lo | (hi << 16);
                }
            }
#pragma unroll
            for (int mi = 0; mi < MT; ++mi) {
                hv[ks][mi][0] = h_piece(mi, k0 + 8 * kh);
                hv[ks][mi][1] = h_piece(mi, k0 + 8 * kh + 4);
            }
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const bool on = 16 * ks < r;
            bf16x8 lf[NI];                      // L2^T fragment: row n, k = 16 ks + 8 kh + 0..7
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const uint4 t = {on ? wds[ks][ni][0] : 0u, on ? wds[ks][ni][1] : 0u, on ? wds[ks][ni][2] : 0u,
                                 on ? wds[ks][ni][3] : 0u};
                lf[ni] = __builtin_bit_cast(bf16x8, t);
            }
#pragma unroll
            for (int mi = 0; mi < MT; ++mi) {
                const float4 h0 = hv[ks][mi][0], h1 = hv[ks][mi][1];
                const float v[8] = {h0.x, h0.y, h0.z, h0.w, h1.x, h1.y, h1.z, h1.w};
                uint32_t hp[4], lp[4];                       // pairs of hi pieces, pairs of lo pieces
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    hp[e] = f2_bf16_rne(v[2 * e], v[2 * e + 1]);
                    lp[e] = f2_bf16_rne(v[2 * e] - bf16lo_f(hp[e]), v[2 * e + 1] - bf16hi_f(hp[e]));
                }
                const uint4 th = {hp[0], hp[1], hp[2], hp[3]};
                const uint4 tl = {lp[0], lp[1], lp[2], lp[3]};
                const uint4 z = {0u, 0u, 0u, 0u};             // an unused k-step multiplies 0 by 0, whatever h holds
                const bf16x8 hhi = __builtin_bit_cast(bf16x8, on ? th : z), hlo = __builtin_bit_cast(bf16x8, on ? tl : z);
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    y[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lf[ni], hhi, y[ni][mi], 0, 0, 0);
                    y[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lf[ni], hlo, y[ni][mi], 0, 0, 0);
                }
            }
        }
    }
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int mi = 0; mi < MT; ++mi) {
                y[ni][mi][4 * q + 0] += bv[ni][q].x;
                y[ni][mi][4 * q + 1] += bv[ni][q].y;
                y[ni][mi][4 * q + 2] += bv[ni][q].z;
                y[ni][mi][4 * q + 3] += bv[ni][q].w;
            }
}

template <int NI, int MT>
__device__ __forceinline__ void add_lowrank_bias(float16v (&y)[NI][MT], const float* __restrict__ h,
                                                 const uint16_t* __restrict__ L2, const float* __restrict__ bias,
                                                 int64_t m0, int n0, int64_t M, int N, int r, int lane) {
    const int l32 = lane & 31;
    add_lowrank_bias_from<NI, MT>(y, [&](const int mi, const int k) {
        int64_t m = m0 + mi * 32 + l32;
        if (m >= M) m = M - 1;
        return *reinterpret_cast<const float4*>(h + m * r + k);
    }, L2, bias, n0, N, r, lane);
}

// The binary32 output (test path): a lane stores 4 consecutive channels of its token per register quad.
template <int NI, int MT>
__device__ __forceinline__ void store_tile_f32(const float16v (&y)[NI][MT], float* __restrict__ yout, int64_t ldy,
                                               int64_t m0, int n0, int64_t M, int lane) {
    const int l32 = lane & 31, kh = lane >> 5;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int n = n0 + ni * 32 + 8 * q + 4 * kh;
#pragma unroll
            for (int mi = 0; mi < MT; ++mi) {
                const int64_t m = m0 + mi * 32 + l32;
                if (m >= M) continue;
                const float4 o = {y[ni][mi][4 * q + 0], y[ni][mi][4 * q + 1], y[ni][mi][4 * q + 2], y[ni][mi][4 * q + 3]};
                *reinterpret_cast<float4*>(yout + m * ldy + n) = o;
            }
        }
}

}  // namespace svdq
