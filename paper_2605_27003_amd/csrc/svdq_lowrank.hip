// Un-fused low-rank branch of eq. 7: h = (x * inv_lambda) L1 and y += h L2.
// Plain binary32 FMA kernels (one thread per output element, coalesced over the
// fast output index).  They exist for callers that run the two halves of the
// layer separately and as an independent cross-check of the fused kernels; the
// fused path does this work on the matrix cores.
#include "svdq_dev.h"
#include "svdq_kernels.h"

namespace svdq {

namespace {

// one block = 8 token rows x r columns; x^ row chunk staged in LDS
__global__ __launch_bounds__(256)
void lowrank_down_kernel(const uint16_t* __restrict__ x, int64_t ldx, const float* __restrict__ inv_lambda,
                         const uint16_t* __restrict__ L1, int64_t M, int K, int r, float* __restrict__ h) {
    constexpr int KC = 512;
    __shared__ float xs[8][KC];
    const int rows = 256 / r;                     // 8 for r = 32, 16 for r = 16 (only 8 used)
    const int j = threadIdx.x % r, rl = threadIdx.x / r;
    const int64_t row0 = (int64_t)blockIdx.x * 8;
    float acc = 0.0f;
    for (int k0 = 0; k0 < K; k0 += KC) {
        for (int e = threadIdx.x; e < 8 * KC; e += 256) {
            int rr = e / KC, kk = e - rr * KC;
            int64_t row = row0 + rr;
            float v = 0.0f;
            if (row < M && k0 + kk < K)
                v = __fmul_rn(bits_f((uint32_t)x[row * ldx + k0 + kk] << 16), inv_lambda[k0 + kk]);
            xs[rr][kk] = v;
        }
        __syncthreads();
        if (rl < 8 && rl < rows) {
            const int kend = (K - k0 < KC) ? (K - k0) : KC;
            for (int kk = 0; kk < kend; ++kk)
                acc = __builtin_fmaf(xs[rl][kk], bits_f((uint32_t)L1[(int64_t)(k0 + kk) * r + j] << 16), acc);
        }
        __syncthreads();
    }
    if (rl < 8 && rl < rows && row0 + rl < M) h[(row0 + rl) * r + j] = acc;
}

__global__ __launch_bounds__(256)
void lowrank_up_kernel(const float* __restrict__ h, const uint16_t* __restrict__ L2, int64_t M, int N, int r,
                       uint16_t* __restrict__ y, int64_t ldy) {
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int64_t m = blockIdx.y;
    if (n >= N || m >= M) return;
    float acc = bits_f((uint32_t)y[m * ldy + n] << 16);
    for (int j = 0; j < r; ++j)
        acc = __builtin_fmaf(h[m * r + j], bits_f((uint32_t)L2[(int64_t)j * N + n] << 16), acc);
    y[m * ldy + n] = (uint16_t)f_bf16_rne(acc);
}

}  // namespace

hipError_t launch_lowrank_down(const void* x, int64_t ldx, const float* inv_lambda, const void* L1,
                               int64_t M, int K, int r, float* h, hipStream_t stream) {
    const unsigned blocks = (unsigned)((M + 7) / 8);
    hipLaunchKernelGGL(lowrank_down_kernel, dim3(blocks), dim3(256), 0, stream,
                       (const uint16_t*)x, ldx, inv_lambda, (const uint16_t*)L1, M, K, r, h);
    return hipGetLastError();
}

hipError_t launch_lowrank_up(const float* h, const void* L2, int64_t M, int N, int r,
                             void* y, int64_t ldy, hipStream_t stream) {
    // gridDim.y is limited to 65535 rows per launch
    for (int64_t m0 = 0; m0 < M; m0 += 65535) {
        const int64_t mc = (M - m0 < 65535) ? (M - m0) : 65535;
        hipLaunchKernelGGL(lowrank_up_kernel, dim3((N + 255) / 256, (unsigned)mc), dim3(256), 0, stream,
                           h + m0 * r, (const uint16_t*)L2, mc, N, r, (uint16_t*)y + m0 * ldy, ldy);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace svdq
