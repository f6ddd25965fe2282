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
// The smoothing factor is folded into the packed L1 operand offline, so the
// matrix cores consume the exact bf16 x; the bit-exact quantiser chain runs in
// binary32 on the vector ALU.
#include "svdq_dev.h"
#include "svdq_kernels.h"

namespace svdq {

namespace {

constexpr int ROWS_PER_BLOCK = 64;
constexpr int WAVES = 4;

// max over the two lanes (l, l^32) that share a token row.  The compiler builtin
// (not inline asm) so that the wait states v_permlane32_swap needs after a VALU
// write of its operands are inserted.
__device__ __forceinline__ float max_pair32(float v) {
    const uint32_t a = f_bits(v);
    auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
    return fmaxf(bits_f(r[0]), bits_f(r[1]));
}

template <bool LOWRANK>
__global__ __launch_bounds__(256, 2)
void quantize_kernel(const uint16_t* __restrict__ x, int64_t ldx,
                     const float* __restrict__ inv_lambda, float rho,
                     const uint4* __restrict__ l1p, int64_t M, int K, int r,
                     uint8_t* __restrict__ qx, float* __restrict__ sx, float* __restrict__ h) {
    __shared__ float hpart[WAVES][ROWS_PER_BLOCK][33];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int rr = lane & 31;          // row inside a 32-row block
    const int hf = lane >> 5;          // which 32-k half of the group
    const int ng = K >> 6;
    const int64_t row0 = (int64_t)blockIdx.x * ROWS_PER_BLOCK;

    float16v acc[2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[b][i] = 0.0f;

    for (int g = wave; g < ng; g += WAVES) {
        // smoothing factors of this lane's 32 k values
        float il[32];
        {
            const float4* pil = reinterpret_cast<const float4*>(inv_lambda + g * 64 + hf * 32);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                float4 t = pil[j];
                il[4 * j + 0] = t.x; il[4 * j + 1] = t.y; il[4 * j + 2] = t.z; il[4 * j + 3] = t.w;
            }
        }
        // B operands (hi and lo piece of inv_lambda*L1) of the four k-steps
        uint4 bfrag[4][2];
        if (LOWRANK) {
            const uint4* pb = l1p + (size_t)g * (4 * 2 * 64) + lane;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                bfrag[s][0] = pb[(s * 2 + 0) * 64];
                bfrag[s][1] = pb[(s * 2 + 1) * 64];
            }
        }
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int64_t row = row0 + 32 * b + rr;
            const int64_t rowc = row < M ? row : M - 1;          // clamp loads of the ragged tail
            const uint4* px = reinterpret_cast<const uint4*>(x + rowc * ldx + g * 64 + hf * 32);
            uint4 xv[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) xv[s] = px[s];

            // eq. 5 in binary32, and the group's reference magnitude
            float xs[32];
            float a = 0.0f;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const uint32_t wds[4] = {xv[s].x, xv[s].y, xv[s].z, xv[s].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float lo = __fmul_rn(bf16lo_f(wds[j]), il[8 * s + 2 * j]);
                    float hi = __fmul_rn(bf16hi_f(wds[j]), il[8 * s + 2 * j + 1]);
                    xs[8 * s + 2 * j] = lo;
                    xs[8 * s + 2 * j + 1] = hi;
                    a = fmaxf(a, fmaxf(fabsf(lo), fabsf(hi)));
                }
            }
            a = max_pair32(a);

            // eq. 8-9: s = (rho * a) / q_max ; zero or denormal scale -> empty group
            float s = __fdiv_rn(__fmul_rn(rho, a), QMAX);
            const bool live = s >= 1.17549435e-38f;
            s = live ? s : 0.0f;
            const float inv = live ? __fdiv_rn(1.0f, s) : 0.0f;

            // eq. 3: clip(rne(x^ * (1/s)), -8, 7).  Clamping before rounding gives the
            // same code; adding 1.5*2^23 rounds to nearest-even and leaves the two's
            // complement integer in the low mantissa bits.
            uint32_t packed[4];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                uint32_t wd = 0;
#pragma unroll
                for (int j = 7; j >= 0; --j) {
                    float u = __fmul_rn(xs[8 * d + j], inv);
                    u = __builtin_amdgcn_fmed3f(u, -8.0f, 7.0f);
                    uint32_t t = f_bits(__fadd_rn(u, 12582912.0f));
                    wd = (wd << 4) | (t & 0xFu);
                }
                packed[d] = wd;
            }
            if (row < M) {
                uint4 o = {packed[0], packed[1], packed[2], packed[3]};
                *reinterpret_cast<uint4*>(qx + row * (int64_t)(K >> 1) + g * 32 + hf * 16) = o;
                if (hf == 0) sx[row * ng + g] = s;
            }

            if (LOWRANK) {
#pragma unroll
                for (int sidx = 0; sidx < 4; ++sidx) {
                    bf16x8 av = __builtin_bit_cast(bf16x8, xv[sidx]);
                    acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8, bfrag[sidx][0]), acc[b], 0, 0, 0);
                    acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8, bfrag[sidx][1]), acc[b], 0, 0, 0);
                }
            }
        }
    }

    if (LOWRANK) {
        // D layout of the 32x32 MFMA: lane holds column (lane % 32); register i holds
        // row 8*(i/4) + 4*(lane/32) + (i%4).
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                int rloc = 32 * b + 8 * (i >> 2) + 4 * hf + (i & 3);
                hpart[wave][rloc][rr] = acc[b][i];
            }
        __syncthreads();
        for (int idx = threadIdx.x; idx < ROWS_PER_BLOCK * r; idx += 256) {
            int rloc = idx / r, j = idx - rloc * r;
            int64_t row = row0 + rloc;
            if (row < M)
                h[row * r + j] = (hpart[0][rloc][j] + hpart[1][rloc][j]) + (hpart[2][rloc][j] + hpart[3][rloc][j]);
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

}  // namespace

hipError_t launch_quantize(const void* x, int64_t ldx, const float* inv_lambda, float rho,
                           const void* l1p, int64_t M, int K, int r,
                           uint8_t* qx, float* sx, float* h, hipStream_t stream) {
    const unsigned blocks = (unsigned)((M + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK);
    if (l1p)
        hipLaunchKernelGGL(quantize_kernel<true>, dim3(blocks), dim3(256), 0, stream,
                           (const uint16_t*)x, ldx, inv_lambda, rho, (const uint4*)l1p, M, K, r, qx, sx, h);
    else
        hipLaunchKernelGGL(quantize_kernel<false>, dim3(blocks), dim3(256), 0, stream,
                           (const uint16_t*)x, ldx, inv_lambda, rho, (const uint4*)nullptr, M, K, r, qx, sx, h);
    return hipGetLastError();
}

hipError_t launch_pack_l1(const void* L1, const float* inv_lambda, int K, int r, void* out, hipStream_t stream) {
    hipLaunchKernelGGL(pack_l1_kernel, dim3(256), dim3(256), 0, stream,
                       (const uint16_t*)L1, inv_lambda, K, r, (uint16_t*)out);
    return hipGetLastError();
}

}  // namespace svdq
