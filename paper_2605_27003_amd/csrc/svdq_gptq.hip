// GPTQ on the residual weights (Sec. III-B: the residual branch of the SVDQuant split is quantised with GPTQ
// instead of round-to-nearest).  Offline calibration, not part of the per-step path: clarity over speed.
//
// The algorithm in its column-sequential form: weights are visited in the order k = 0..K-1; a visited weight is
// rounded to the int4 grid of its (channel, 64-group) scale and its rounding error is spread over the not yet
// visited weights of the same channel in proportion to row k of the inverse Hessian of the layer-wise objective
// ||X^ (R - R^)||^2 (H = X^T X^ plus damping), from which index k is then eliminated.  Everything runs in
// binary64 with one explicitly rounded operation per arithmetic step and no reductions other than max and one
// sequential sum, so that a CPU reference repeats every bit.  The published implementation factors H^-1 once
// (Cholesky) and reads the same numbers off the factor; this form trades that for elementwise kernels:
// K^3 / 3 updates of H^-1 and K^2 N / 2 updates of the weights, about a second for a 5120 x 5120 layer.
#include "svdq_dev.h"
#include "svdq_kernels.h"

namespace svdq {

namespace {

// ---- H += X^T X^, X^ = x * inv_lambda in binary32 (eq. 5), products and sums in binary64
constexpr int HT = 64;   // tile of H per block
__global__ __launch_bounds__(256)
void hessian_kernel(const uint16_t* __restrict__ x, int64_t ldx, const float* __restrict__ inv_lambda,
                    int64_t M, int K, double* __restrict__ H) {
    __shared__ double xa[16][HT + 1], xb[16][HT + 1];
    const int a0 = blockIdx.y * HT, b0 = blockIdx.x * HT;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    double acc[4][4] = {};
    for (int64_t m0 = 0; m0 < M; m0 += 16) {
        for (int e = threadIdx.x; e < 16 * HT; e += 256) {
            const int mr = e / HT, c = e - mr * HT;
            const int64_t m = m0 + mr;
            double va = 0.0, vb = 0.0;
            if (m < M) {
                if (a0 + c < K) va = (double)__fmul_rn(bits_f((uint32_t)x[m * ldx + a0 + c] << 16), inv_lambda[a0 + c]);
                if (b0 + c < K) vb = (double)__fmul_rn(bits_f((uint32_t)x[m * ldx + b0 + c] << 16), inv_lambda[b0 + c]);
            }
            xa[mr][c] = va;
            xb[mr][c] = vb;
        }
        __syncthreads();
#pragma unroll
        for (int mr = 0; mr < 16; ++mr)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __fma_rn(xa[mr][ty * 4 + i], xb[mr][tx * 4 + j], acc[i][j]);
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int a = a0 + ty * 4 + i, b = b0 + tx * 4 + j;
            if (a < K && b < K) H[(size_t)a * K + b] += acc[i][j];
        }
}

// ---- preparation: binary64 copies, dead channels, damping with the diagonal summed in index order
__global__ void prepare_kernel(const float* __restrict__ R, const double* __restrict__ H, double damp, int N, int K,
                               double* __restrict__ A, double* __restrict__ W) {
    const size_t stride = (size_t)gridDim.x * blockDim.x, t0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    __shared__ double add;
    if (threadIdx.x == 0) {
        double s = 0.0;
        for (int k = 0; k < K; ++k) {
            const double d = H[(size_t)k * K + k];
            s = __dadd_rn(s, d == 0.0 ? 1.0 : d);
        }
        add = __dmul_rn(damp, __ddiv_rn(s, (double)K));
    }
    __syncthreads();
    for (size_t e = t0; e < (size_t)K * K; e += stride) {
        const int a = (int)(e / K), b = (int)(e - (size_t)a * K);
        double v = H[e];
        if (a == b) v = __dadd_rn(v == 0.0 ? 1.0 : v, add);
        A[e] = v;
    }
    for (size_t e = t0; e < (size_t)K * N; e += stride) {
        const int k = (int)(e / N);
        W[e] = (H[(size_t)k * K + k] == 0.0) ? 0.0 : (double)R[e];
    }
}

// ---- in-place Gauss-Jordan inverse without pivoting, step p
__global__ void gj_pivot_kernel(const double* __restrict__ A, int K, int p, double* __restrict__ col, double* __restrict__ row) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= K) return;
    const double d = A[(size_t)p * K + p];
    col[i] = A[(size_t)i * K + p];
    row[i] = __ddiv_rn(A[(size_t)p * K + i], d);
}
__global__ void gj_update_kernel(double* __restrict__ A, int K, int p, const double* __restrict__ col, const double* __restrict__ row) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const double d = col[p];
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < (size_t)K * K; e += stride) {
        const int a = (int)(e / K), j = (int)(e - (size_t)a * K);
        double v;
        if (a == p) v = (j == p) ? __ddiv_rn(1.0, d) : row[j];
        else if (j == p) v = __ddiv_rn(-col[a], d);
        else v = __dsub_rn(A[e], __dmul_rn(col[a], row[j]));
        A[e] = v;
    }
}

// ---- column i: scale at a group start, code, error
__global__ void column_kernel(const double* __restrict__ W, const double* __restrict__ Hinv, int N, int K, int i,
                              float* __restrict__ scur, float* __restrict__ sw, int8_t* __restrict__ codes,
                              double* __restrict__ err) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    float s;
    if ((i & 63) == 0) {
        double a = 0.0;
        for (int t = 0; t < 64; ++t) a = fmax(a, fabs(W[(size_t)(i + t) * N + n]));
        s = __fdiv_rn((float)a, 7.0f);
        scur[n] = s;
        sw[(size_t)(i >> 6) * N + n] = s;
    } else {
        s = scur[n];
    }
    const double w = W[(size_t)i * N + n];
    float q = 0.0f;
    if (s > 0.0f) q = fminf(fmaxf(rintf(__fdiv_rn((float)w, s)), -8.0f), 7.0f);
    codes[(size_t)i * N + n] = (int8_t)q;
    err[n] = __ddiv_rn(__dsub_rn(w, __dmul_rn((double)q, (double)s)), Hinv[(size_t)i * K + i]);
}
// ---- spread the error over the weights not yet visited
__global__ void spread_kernel(double* __restrict__ W, const double* __restrict__ Hinv, const double* __restrict__ err,
                              int N, int K, int i) {
    const size_t total = (size_t)(K - 1 - i) * N, stride = (size_t)gridDim.x * blockDim.x;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
        const int j = i + 1 + (int)(e / N), n = (int)(e % N);
        W[(size_t)j * N + n] = __dsub_rn(W[(size_t)j * N + n], __dmul_rn(Hinv[(size_t)i * K + j], err[n]));
    }
}
// ---- eliminate index i from the inverse Hessian
__global__ void eliminate_kernel(double* __restrict__ Hinv, int K, int i) {
    const int rem = K - 1 - i;
    const size_t total = (size_t)rem * rem, stride = (size_t)gridDim.x * blockDim.x;
    const double d = Hinv[(size_t)i * K + i];
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
        const int a = i + 1 + (int)(e / rem), b = i + 1 + (int)(e % rem);
        const double t = __ddiv_rn(Hinv[(size_t)i * K + b], d);
        Hinv[(size_t)a * K + b] = __dsub_rn(Hinv[(size_t)a * K + b], __dmul_rn(Hinv[(size_t)a * K + i], t));
    }
}
// ---- codes [K][N] -> canonical qw [N][K/2] (low nibble = even k)
__global__ void pack_codes_kernel(const int8_t* __restrict__ codes, int N, int K, uint8_t* __restrict__ qw) {
    const size_t total = (size_t)N * (K / 2), stride = (size_t)gridDim.x * blockDim.x;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
        const int n = (int)(e / (K / 2)), k2 = (int)(e % (K / 2));
        const uint32_t lo = (uint32_t)codes[(size_t)(2 * k2) * N + n] & 15u, hi = (uint32_t)codes[(size_t)(2 * k2 + 1) * N + n] & 15u;
        qw[e] = (uint8_t)(lo | (hi << 4));
    }
}

inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }
inline unsigned blocks_for(size_t n) { size_t b = (n + 255) / 256; return (unsigned)(b < 1 ? 1 : (b > 4096 ? 4096 : b)); }

}  // namespace

size_t gptq_workspace_bytes(int N, int K) {
    return up256((size_t)K * K * 8) + up256((size_t)K * N * 8) + up256((size_t)N * 8) + up256((size_t)N * 4) +
           2 * up256((size_t)K * 8) + up256((size_t)K * N);
}

hipError_t launch_gptq_hessian(const void* x, int64_t ldx, const float* inv_lambda, int64_t M, int K, double* H,
                               hipStream_t stream) {
    const unsigned t = (unsigned)((K + HT - 1) / HT);
    hipLaunchKernelGGL(hessian_kernel, dim3(t, t), dim3(256), 0, stream, (const uint16_t*)x, ldx, inv_lambda, M, K, H);
    return hipGetLastError();
}

hipError_t launch_gptq_quantize(const float* R, const double* H, double damp, int N, int K, void* workspace,
                                uint8_t* qw, float* sw, hipStream_t stream) {
    uint8_t* p = (uint8_t*)workspace;
    double* A = (double*)p;        p += up256((size_t)K * K * 8);
    double* W = (double*)p;        p += up256((size_t)K * N * 8);
    double* err = (double*)p;      p += up256((size_t)N * 8);
    float* scur = (float*)p;       p += up256((size_t)N * 4);
    double* col = (double*)p;      p += up256((size_t)K * 8);
    double* row = (double*)p;      p += up256((size_t)K * 8);
    int8_t* codes = (int8_t*)p;
    hipLaunchKernelGGL(prepare_kernel, dim3(1024), dim3(256), 0, stream, R, H, damp, N, K, A, W);
    for (int q = 0; q < K; ++q) {
        hipLaunchKernelGGL(gj_pivot_kernel, dim3((K + 255) / 256), dim3(256), 0, stream, A, K, q, col, row);
        hipLaunchKernelGGL(gj_update_kernel, dim3(blocks_for((size_t)K * K)), dim3(256), 0, stream, A, K, q, col, row);
    }
    for (int i = 0; i < K; ++i) {
        hipLaunchKernelGGL(column_kernel, dim3((N + 255) / 256), dim3(256), 0, stream, W, A, N, K, i, scur, sw, codes, err);
        if (i + 1 < K) {
            hipLaunchKernelGGL(spread_kernel, dim3(blocks_for((size_t)(K - 1 - i) * N)), dim3(256), 0, stream, W, A, err, N, K, i);
            hipLaunchKernelGGL(eliminate_kernel, dim3(blocks_for((size_t)(K - 1 - i) * (K - 1 - i))), dim3(256), 0, stream, A, K, i);
        }
    }
    hipLaunchKernelGGL(pack_codes_kernel, dim3(blocks_for((size_t)N * (K / 2))), dim3(256), 0, stream, codes, N, K, qw);
    return hipGetLastError();
}

}  // namespace svdq
