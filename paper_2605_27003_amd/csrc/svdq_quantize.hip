// Kernel (a): one HBM pass over x that smooths (eq. 5), takes the per-token
// per-64-group absmax, derives the clipped scale (eq. 8-9), rounds and packs
// int4 codes (eq. 3) and feeds the raw bf16 x to the bf16 matrix cores for the
// low-rank down-projection h = x^ L1 (eq. 7).
//
// Layout.  A block of 256 threads (4 waves) owns 64 token rows; wave w owns the
// 64-groups g = w, w+4, ...  Lane l of a wave holds row (l % 32) of a 32-row
// block and the 32 consecutive k values [64 g + 32 (l/32), +32) of that row:
// 64 contiguous bytes, read as four 16-byte loads.  That is at the same time
//   - the A-operand layout of v_mfma_f32_32x32x16_bf16 (row = lane % 32, eight
//     k per lane and k-step), so x goes to the matrix cores without a shuffle;
//   - a layout in which the absmax of a group needs one cross-lane exchange
//     (lanes l and l^32) and a lane packs 16 contiguous bytes of codes.
// Outputs are group-major (qx[g][row][32 B], sx[g][row]): what a wave produces for
// one group and 32 rows is 1 KB of codes and 128 B of scales, contiguous, and it is
// also the order in which the GEMM stages them.
// The smoothing factor is folded into the packed L1 operand offline, so the
// matrix cores consume the exact bf16 x; the bit-exact quantiser chain runs in
// binary32 on the vector ALU.
#include "svdq_act.h"
#include "svdq_dev.h"
#include "svdq_kernels.h"
#include "svdq_lds.h"
#include "svdq_quant_dev.h"

namespace svdq {

namespace {

constexpr int ROWS_PER_BLOCK = 64;
constexpr int WAVES = 4;

constexpr int HPART_BYTES = WAVES * ROWS_PER_BLOCK * 33 * 4;

// E3M2 = false: qx [K/64][M][32 B] nibbles.  E3M2 = true: qx is the activation operand buffer of the FP6 GEMM,
// per group a block of Mp rows (Mp = M rounded up to a multiple of 4; rows M..Mp-1 are never written):
//   [Mp][2 halves][16 B]   bytes 0..15 of each lane's 24 code bytes
//   [2 halves][Mp][8 B]    bytes 16..23
//   [Mp] x 8 B             the token scale as two bf16 pieces, p = hi | lo << 16, stored twice ({p, p} is the
//                          m-side operand of the scale-product MFMA)
// sx [K/64][M] binary32 is written in both cases (skipped if null with E3M2).
// GELU = true: x is the feed-forward block's pre-activation; every value is replaced by bf16(gelu(x)) as it
// arrives (svdq_act.h), and the pass continues as if a separate element-wise kernel had written that tensor.
template <bool LOWRANK, bool E3M2, bool GELU>
__global__ __launch_bounds__(256, 2)
void quantize_kernel(const uint16_t* __restrict__ x, int64_t ldx,
                     const float* __restrict__ inv_lambda, float rho,
                     const uint4* __restrict__ l1p, int64_t M, int K, int r,
                     uint8_t* __restrict__ qx, float* __restrict__ sx, float* __restrict__ h) {
    // LDS: inv_lambda[K] during the main loop, then the 4 x 64 x 33 partial sums of h
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    float* il_s = reinterpret_cast<float*>(smem_raw);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int rr = lane & 31;          // row inside a 32-row block
    const int hf = lane >> 5;          // which 32-k half of the group
    const int ng = K >> 6;
    const int64_t row0 = (int64_t)blockIdx.x * ROWS_PER_BLOCK;

    for (int i = tid * 4; i < K; i += 1024)
        *reinterpret_cast<float4*>(il_s + i) = *reinterpret_cast<const float4*>(inv_lambda + i);

    float16v acc[2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[b][i] = 0.0f;

    const uint16_t* xrow[2];
    int64_t rows[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        rows[b] = row0 + 32 * b + rr;
        const int64_t rowc = rows[b] < M ? rows[b] : M - 1;             // clamp loads of the ragged tail
        xrow[b] = x + rowc * ldx + hf * 32;
    }

    // software pipeline: x of this wave's NEXT group is in flight while the current one is processed.
    // Two register buffers alternate roles (the round body is instantiated twice), so there is no copy
    // and the wait for a prefetched group sits right before its first use, one full round later.
    uint4 xa[2][4], xb[2][4];
    if (wave < ng) {
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int s = 0; s < 4; ++s) xa[b][s] = reinterpret_cast<const uint4*>(xrow[b] + wave * 64)[s];
    }
    __syncthreads();

    const int rounds = (ng + WAVES - 1) / WAVES;
    auto round_body = [&](const int rd, uint4 (&xc)[2][4], uint4 (&xn)[2][4]) {
        const int g = rd * WAVES + wave;
        if (g < ng) {
            // B operands (hi and lo piece of inv_lambda*L1) of the four k-steps: issued first, used last
            uint4 bfrag[4][2];
            if (LOWRANK) {
                const uint4* pb = l1p + (size_t)g * (4 * 2 * 64) + lane;
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    bfrag[s][0] = pb[(s * 2 + 0) * 64];
                    bfrag[s][1] = pb[(s * 2 + 1) * 64];
                }
            }
            // keep the L2-resident operand loads ahead of the HBM prefetch in program order: the
            // matrix-core step then waits for them without draining the prefetch (vmcnt counts in order)
            __builtin_amdgcn_sched_barrier(0);
            // unconditional (the last round re-reads its own group): a load under a branch would make
            // the compiler assume the smaller outstanding count and wait for the prefetch early
            const int gn = (g + WAVES < ng) ? g + WAVES : g;
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int s = 0; s < 4; ++s) xn[b][s] = reinterpret_cast<const uint4*>(xrow[b] + gn * 64)[s];
            __builtin_amdgcn_sched_barrier(0);

            const float* il_lds = il_s + g * 64 + hf * 32;
            if (GELU) {
#pragma unroll
                for (int b = 0; b < 2; ++b) gelu_tanh_rows(xc[b]);
            }
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                LaneCodes<E3M2> codes;
                float s;
                quantize_rows<E3M2>(xc[b], il_lds, rho, codes, s);
                // group-major outputs: the 32 rows of this block are 1 KB of codes and 128 B of scales, contiguous
                if (rows[b] < M) {
                    if constexpr (E3M2) {
                        const size_t Mp = (size_t)((M + 3) & ~(int64_t)3);
                        uint8_t* blk = qx + (size_t)g * Mp * E3M2_ROW_BYTES;
                        *reinterpret_cast<uint4*>(blk + (size_t)rows[b] * 32 + hf * 16) = codes.lo;
                        *reinterpret_cast<uint2*>(blk + Mp * 32 + ((size_t)hf * Mp + rows[b]) * 8) = codes.hi;
                        if (hf == 0) {
                            const uint32_t p = split_bf16(s);
                            *reinterpret_cast<uint2*>(blk + Mp * 48 + (size_t)rows[b] * 8) = uint2{p, p};
                            if (sx) sx[(size_t)g * M + rows[b]] = s;
                        }
                    } else {
                        *reinterpret_cast<uint4*>(qx + ((size_t)g * M + rows[b]) * 32 + hf * 16) = codes.lo;
                        if (hf == 0) sx[(size_t)g * M + rows[b]] = s;
                    }
                }
            }
            if (LOWRANK) {
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int sidx = 0; sidx < 4; ++sidx) {
                        bf16x8 av = __builtin_bit_cast(bf16x8, xc[b][sidx]);
                        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8, bfrag[sidx][0]), acc[b], 0, 0, 0);
                        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8, bfrag[sidx][1]), acc[b], 0, 0, 0);
                    }
            }
        }
    };
    for (int rd = 0; rd < rounds; rd += 2) {
        round_body(rd, xa, xb);
        if (rd + 1 < rounds) round_body(rd + 1, xb, xa);
    }

    if (LOWRANK) {
        // D layout of the 32x32 MFMA: lane holds column (lane % 32); register i holds
        // row 8*(i/4) + 4*(lane/32) + (i%4).
        __syncthreads();                                     // every wave is done with inv_lambda in LDS
        float* hpart = reinterpret_cast<float*>(smem_raw);   // [WAVES][64][33]
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                int rloc = 32 * b + 8 * (i >> 2) + 4 * hf + (i & 3);
                hpart[(wave * ROWS_PER_BLOCK + rloc) * 33 + rr] = acc[b][i];
            }
        __syncthreads();
        for (int idx = tid; idx < ROWS_PER_BLOCK * r; idx += 256) {
            int rloc = idx / r, j = idx - rloc * r;
            int64_t row = row0 + rloc;
            if (row < M)
                h[row * r + j] = (hpart[(0 * ROWS_PER_BLOCK + rloc) * 33 + j] + hpart[(1 * ROWS_PER_BLOCK + rloc) * 33 + j]) +
                                 (hpart[(2 * ROWS_PER_BLOCK + rloc) * 33 + j] + hpart[(3 * ROWS_PER_BLOCK + rloc) * 33 + j]);
        }
    }
}

// rn(inv_lambda[k] * L1[k,j]) split into hi + lo bf16, in B-operand order of
// v_mfma_f32_32x32x16_bf16 matched to the A layout above: fragment (g, s, piece)
// is 64 lanes x 8 bf16; lane (j = lane % 32, hf = lane / 32) element i holds
// k = 64 g + 32 hf + 8 s + i, column j (zero for j >= r).
__global__ void pack_l1_kernel(const uint16_t* __restrict__ L1, const float* __restrict__ inv_lambda,
                               int K, int r, uint16_t* __restrict__ out) {
    const int64_t total = (int64_t)(K >> 6) * 4 * 64 * 8;          // elements per piece over all fragments
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        int i = (int)(e & 7);
        int lane = (int)((e >> 3) & 63);
        int s = (int)((e >> 9) & 3);
        int g = (int)(e >> 11);
        int j = lane & 31, hf = lane >> 5;
        int k = 64 * g + 32 * hf + 8 * s + i;
        float v = 0.0f;
        if (j < r) v = __fmul_rn(bits_f((uint32_t)L1[(int64_t)k * r + j] << 16), inv_lambda[k]);
        uint32_t hi = f_bf16_rne(v);
        float rem = __fsub_rn(v, bits_f(hi << 16));
        uint32_t lo = f_bf16_rne(rem);
        size_t base = ((size_t)(g * 4 + s) * 2) * 512 + (size_t)lane * 8 + i;
        out[base] = (uint16_t)hi;
        out[base + 512] = (uint16_t)lo;
    }
}

// Test hook: the scalar part of the quantiser chain (eq. 8-9) on arbitrary inputs, through the same
// device functions the quantise kernel uses.
__global__ void scale_chain_kernel(const float* __restrict__ a, float rho, int64_t n,
                                   float* __restrict__ s_out, float* __restrict__ inv_out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float s = div7(__fmul_rn(rho, a[i]));
    const bool live = s >= 1.17549435e-38f;
    s = live ? s : 0.0f;
    s_out[i] = s;
    inv_out[i] = live ? recip_rn(s) : 0.0f;
}

}  // namespace

hipError_t launch_scale_chain(const float* a, float rho, int64_t n, float* s, float* inv, hipStream_t stream) {
    const int64_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(scale_chain_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, a, rho, n, s, inv);
    return hipGetLastError();
}

template <bool E3M2, bool GELU>
static hipError_t launch_quantize_any(const void* x, int64_t ldx, const float* inv_lambda, float rho,
                                      const void* l1p, int64_t M, int K, int r,
                                      uint8_t* qx, float* sx, float* h, hipStream_t stream) {
    const unsigned blocks = (unsigned)((M + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK);
    size_t lds = (size_t)K * sizeof(float);
    if (lds < (size_t)HPART_BYTES) lds = HPART_BYTES;
    if (l1p)
        hipLaunchKernelGGL((quantize_kernel<true, E3M2, GELU>), dim3(blocks), dim3(256), lds, stream,
                           (const uint16_t*)x, ldx, inv_lambda, rho, (const uint4*)l1p, M, K, r, qx, sx, h);
    else
        hipLaunchKernelGGL((quantize_kernel<false, E3M2, GELU>), dim3(blocks), dim3(256), lds, stream,
                           (const uint16_t*)x, ldx, inv_lambda, rho, (const uint4*)nullptr, M, K, r, qx, sx, h);
    return hipGetLastError();
}

hipError_t launch_quantize(const void* x, int64_t ldx, const float* inv_lambda, float rho,
                           const void* l1p, int64_t M, int K, int r,
                           uint8_t* qx, float* sx, float* h, bool gelu, hipStream_t stream) {
    return gelu ? launch_quantize_any<false, true>(x, ldx, inv_lambda, rho, l1p, M, K, r, qx, sx, h, stream)
                : launch_quantize_any<false, false>(x, ldx, inv_lambda, rho, l1p, M, K, r, qx, sx, h, stream);
}

hipError_t launch_quantize_e3m2(const void* x, int64_t ldx, const float* inv_lambda, float rho,
                                const void* l1p, int64_t M, int K, int r,
                                uint8_t* act, float* sx, float* h, bool gelu, hipStream_t stream) {
    return gelu ? launch_quantize_any<true, true>(x, ldx, inv_lambda, rho, l1p, M, K, r, act, sx, h, stream)
                : launch_quantize_any<true, false>(x, ldx, inv_lambda, rho, l1p, M, K, r, act, sx, h, stream);
}

// Test hook: the activation alone, through the device function the quantise kernels use.
__global__ void gelu_kernel(const uint16_t* __restrict__ x, int64_t n, uint16_t* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = (uint16_t)f_bf16_rne(gelu_tanh_f32(bits_f((uint32_t)x[i] << 16)));
}

hipError_t launch_gelu(const void* x, int64_t n, void* out, hipStream_t stream) {
    hipLaunchKernelGGL(gelu_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, (const uint16_t*)x, n, (uint16_t*)out);
    return hipGetLastError();
}

hipError_t launch_pack_l1(const void* L1, const float* inv_lambda, int K, int r, void* out, hipStream_t stream) {
    hipLaunchKernelGGL(pack_l1_kernel, dim3(256), dim3(256), 0, stream,
                       (const uint16_t*)L1, inv_lambda, K, r, (uint16_t*)out);
    return hipGetLastError();
}

}  // namespace svdq
