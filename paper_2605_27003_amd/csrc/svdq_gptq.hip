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
// K^3 updates for the inverse, K^3 / 3 of H^-1 and K^2 N / 2 of the weights during the visit, taken in panels of 64
// pivots (below) so that the matrices cross HBM once per panel.
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

// ---- Panel-blocked form of both eliminations.  Every element of H^-1 (and of W) must receive, in the order of the
// pivots, one rounded product and one rounded subtraction per pivot: that sequence per element is the definition, and
// it does not say WHEN an element is touched.  Pivots are taken in panels of PB = 64.  Inside a panel only the panel's
// own rows and columns (2 x 64 x K elements) are brought up to date after every pivot, by small kernels, and each
// pivot's column (as it stood when the pivot was taken) and scaled row are saved; everything else receives its 64
// updates in one pass at the end of the panel from the saved columns and rows, in pivot order, with the same two
// rounded operations per update.  Bit-identical to the pivot-by-pivot form; the K x K matrix crosses HBM once per
// panel instead of once per pivot.
constexpr int PB = 64;

// X[a][b] <- (..((X[a][b] - L[a][0] R[0][b]) - L[a][1] R[1][b]).. - L[a][PB-1] R[PB-1][b]) for a in [a0, a1),
// b in [b0, b1), skipping the 64-aligned index block [skip, skip + PB) in both directions (skip < 0: none).
// L is [rows][PB], R is [PB][ldr].  a0, a1, b0 multiples of 64.  One 64 x 64 tile per block, 4 x 4 elements per thread.
__global__ __launch_bounds__(256)
void seq_rank_update_kernel(double* __restrict__ X, size_t ldx, int a0, int a1, int b0, int b1, int skip,
                            const double* __restrict__ L, const double* __restrict__ R, size_t ldr) {
    __shared__ double Lt[PB][64];       // Lt[q][row]
    __shared__ double Rs[PB][64];       // Rs[q][col]
    const int ta = a0 + blockIdx.y * 64, tb = b0 + blockIdx.x * 64;
    if (ta == skip || tb == skip) return;
    for (int e = threadIdx.x; e < 64 * PB; e += 256) {
        const int rr = e / PB, q = e - rr * PB;
        Lt[q][rr] = (ta + rr < a1) ? L[(size_t)(ta + rr) * PB + q] : 0.0;
        const int qq = e / 64, c = e - qq * 64;
        Rs[qq][c] = (tb + c < b1) ? R[(size_t)qq * ldr + tb + c] : 0.0;
    }
    __syncthreads();
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    double v[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int a = ta + ty * 4 + i, c = tb + tx * 4 + j;
            v[i][j] = (a < a1 && c < b1) ? X[(size_t)a * ldx + c] : 0.0;
        }
    for (int q = 0; q < PB; ++q) {
        double l[4], r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) l[i] = Lt[q][ty * 4 + i];
#pragma unroll
        for (int j = 0; j < 4; ++j) r[j] = Rs[q][tx * 4 + j];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) v[i][j] = __dsub_rn(v[i][j], __dmul_rn(l[i], r[j]));
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int a = ta + ty * 4 + i, c = tb + tx * 4 + j;
            if (a < a1 && c < b1) X[(size_t)a * ldx + c] = v[i][j];
        }
}

// ---- in-place Gauss-Jordan inverse without pivoting.  Step p: d = A[p][p], col = A[:, p], row = A[p, :] / d;
// A[a][j] -= col[a] row[j] elsewhere, A[p][j] = row[j], A[a][p] = -col[a] / d, A[p][p] = 1 / d.
// gj_pivot: save col and row of pivot p (panel starting at p0) as they stand.
__global__ void gj_pivot_kernel(const double* __restrict__ A, int K, int p, int p0, double* __restrict__ C, double* __restrict__ Rw) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= K) return;
    const double d = A[(size_t)p * K + p];
    C[(size_t)i * PB + (p - p0)] = A[(size_t)i * K + p];
    Rw[(size_t)(p - p0) * K + i] = __ddiv_rn(A[(size_t)p * K + i], d);
}
// gj_panel: apply step p to the panel's columns (all rows) and the panel's rows (all other columns)
__global__ void gj_panel_kernel(double* __restrict__ A, int K, int p, int p0, const double* __restrict__ C, const double* __restrict__ Rw) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const int q = p - p0;
    const double d = C[(size_t)p * PB + q];
    const size_t n1 = (size_t)K * PB, total = n1 + (size_t)PB * (K - PB);
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
        int a, j;
        if (e < n1) {                                   // the panel's columns
            a = (int)(e / PB);
            j = p0 + (int)(e - (size_t)a * PB);
        } else {                                        // the panel's rows, columns outside the panel
            const size_t f = e - n1;
            a = p0 + (int)(f / (K - PB));
            j = (int)(f - (size_t)(a - p0) * (K - PB));
            if (j >= p0) j += PB;
        }
        const size_t at = (size_t)a * K + j;
        double v;
        if (a == p) v = (j == p) ? __ddiv_rn(1.0, d) : Rw[(size_t)q * K + j];
        else if (j == p) v = __ddiv_rn(-C[(size_t)a * PB + q], d);
        else v = __dsub_rn(A[at], __dmul_rn(C[(size_t)a * PB + q], Rw[(size_t)q * K + j]));
        A[at] = v;
    }
}

// ---- column i: scale at a group start, code, error (kept in Err[i - i0][:] for the deferred spreading)
__global__ void column_kernel(const double* __restrict__ W, const double* __restrict__ Hinv, int N, int K, int i, int i0,
                              float* __restrict__ scur, float* __restrict__ sw, int8_t* __restrict__ codes,
                              double* __restrict__ Err) {
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
    Err[(size_t)(i - i0) * N + n] = __ddiv_rn(__dsub_rn(w, __dmul_rn((double)q, (double)s)), Hinv[(size_t)i * K + i]);
}
// ---- spread the error of column i over the panel's not yet visited weights (rows i + 1 .. i0 + PB - 1)
__global__ void spread_panel_kernel(double* __restrict__ W, const double* __restrict__ Hinv, const double* __restrict__ Err,
                                    int N, int K, int i, int i0) {
    const size_t total = (size_t)(i0 + PB - 1 - i) * N, stride = (size_t)gridDim.x * blockDim.x;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
        const int j = i + 1 + (int)(e / N), n = (int)(e % N);
        W[(size_t)j * N + n] = __dsub_rn(W[(size_t)j * N + n], __dmul_rn(Hinv[(size_t)i * K + j], Err[(size_t)(i - i0) * N + n]));
    }
}
// ---- eliminate index i from the inverse Hessian inside the panel: Hinv[a][b] -= Hinv[a][i] (Hinv[i][b] / d) for
// a, b > i with a or b in the panel; row i, scaled row i and column i are saved for the deferred updates
// (HrowT[j][q] = Hinv[i][j], T[q][b] = Hinv[i][b] / d, Hc[a][q] = Hinv[a][i]); row and column i are not written.
__global__ void eliminate_panel_kernel(double* __restrict__ Hinv, int K, int i, int i0,
                                       double* __restrict__ HrowT, double* __restrict__ T, double* __restrict__ Hc) {
    const size_t stride = (size_t)gridDim.x * blockDim.x, t0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int q = i - i0, i1 = i0 + PB;
    const double d = Hinv[(size_t)i * K + i];
    for (size_t e = t0; e < (size_t)K; e += stride) {
        const int j = (int)e;
        const double hij = Hinv[(size_t)i * K + j];
        HrowT[(size_t)j * PB + q] = hij;
        T[(size_t)q * K + j] = __ddiv_rn(hij, d);
        Hc[(size_t)j * PB + q] = Hinv[(size_t)j * K + i];
    }
    const int rp = i1 - 1 - i;                          // panel rows / columns still alive after i
    const int rem = K - 1 - i;                          // indices > i
    const size_t n1 = (size_t)rp * rem, total = n1 + (size_t)(K - i1) * rp;
    for (size_t e = t0; e < total; e += stride) {
        int a, b;
        if (e < n1) {                                   // rows of the panel, every column > i
            a = i + 1 + (int)(e / rem);
            b = i + 1 + (int)(e % rem);
        } else {                                        // rows below the panel, columns of the panel
            const size_t f = e - n1;
            a = i1 + (int)(f / rp);
            b = i + 1 + (int)(f % rp);
        }
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
    return up256((size_t)K * K * 8) + up256((size_t)K * N * 8) + up256((size_t)N * 4) + up256((size_t)K * N) +
           4 * up256((size_t)K * PB * 8) + up256((size_t)PB * N * 8);
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
    float* scur = (float*)p;       p += up256((size_t)N * 4);
    int8_t* codes = (int8_t*)p;    p += up256((size_t)K * N);
    double* Lc = (double*)p;       p += up256((size_t)K * PB * 8);     // saved pivot columns      [K][PB]
    double* Rr = (double*)p;       p += up256((size_t)K * PB * 8);     // saved scaled pivot rows  [PB][K]
    double* HrowT = (double*)p;    p += up256((size_t)K * PB * 8);     // saved rows of H^-1       [K][PB]
    double* Hc = (double*)p;       p += up256((size_t)K * PB * 8);     // saved columns of H^-1    [K][PB]
    double* Err = (double*)p;                                          // errors of the panel      [PB][N]
    const dim3 tilesKK((unsigned)(K / 64), (unsigned)(K / 64));
    hipLaunchKernelGGL(prepare_kernel, dim3(1024), dim3(256), 0, stream, R, H, damp, N, K, A, W);
    for (int p0 = 0; p0 < K; p0 += PB) {               // Gauss-Jordan, one panel of pivots at a time
        for (int q = p0; q < p0 + PB; ++q) {
            hipLaunchKernelGGL(gj_pivot_kernel, dim3((K + 255) / 256), dim3(256), 0, stream, A, K, q, p0, Lc, Rr);
            hipLaunchKernelGGL(gj_panel_kernel, dim3(blocks_for((size_t)K * PB * 2)), dim3(256), 0, stream, A, K, q, p0, Lc, Rr);
        }
        if (K > PB)
            hipLaunchKernelGGL(seq_rank_update_kernel, tilesKK, dim3(256), 0, stream, A, (size_t)K, 0, K, 0, K, p0, Lc, Rr, (size_t)K);
    }
    for (int i0 = 0; i0 < K; i0 += PB) {               // the weights, one panel (= one 64-group) at a time
        const int i1 = i0 + PB;
        for (int i = i0; i < i1; ++i) {
            hipLaunchKernelGGL(column_kernel, dim3((N + 255) / 256), dim3(256), 0, stream, W, A, N, K, i, i0, scur, sw, codes, Err);
            if (i + 1 < i1)
                hipLaunchKernelGGL(spread_panel_kernel, dim3(blocks_for((size_t)(i1 - 1 - i) * N)), dim3(256), 0, stream, W, A, Err, N, K, i, i0);
            if (i1 < K || i + 1 < i1)
                hipLaunchKernelGGL(eliminate_panel_kernel, dim3(blocks_for((size_t)K * PB)), dim3(256), 0, stream, A, K, i, i0, HrowT, Rr, Hc);
        }
        if (i1 < K) {                                   // the deferred updates of everything behind the panel
            const int rest = K - i1;
            hipLaunchKernelGGL(seq_rank_update_kernel, dim3((unsigned)((N + 63) / 64), (unsigned)(rest / 64)), dim3(256), 0, stream,
                               W, (size_t)N, i1, K, 0, N, -1, HrowT, Err, (size_t)N);
            hipLaunchKernelGGL(seq_rank_update_kernel, dim3((unsigned)(rest / 64), (unsigned)(rest / 64)), dim3(256), 0, stream,
                               A, (size_t)K, i1, K, i1, K, -1, Hc, Rr, (size_t)K);
        }
    }
    hipLaunchKernelGGL(pack_codes_kernel, dim3(blocks_for((size_t)N * (K / 2))), dim3(256), 0, stream, codes, N, K, qw);
    return hipGetLastError();
}

}  // namespace svdq
