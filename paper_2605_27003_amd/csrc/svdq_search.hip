// Reconstruction error of the clipping-ratio search (Sec. III-C, the arg-min objective over the candidate
// set): sum over a layer output of (Y - Y^)^2, Y the full-precision layer output and Y^ the quantised
// layer's, both bf16 [M, N].  The search itself runs the hot-path kernels once per candidate ratio and
// compares these sums; this file is the one extra kernel it needs.
//
// Deterministic: NPART blocks each own a fixed, strided set of 8-element chunks and sum them in a fixed
// order in binary64; a second one-block kernel adds the NPART partial sums in index order.
//
// Also here: the expectation over a bin's calibration steps (the same reduction ADDED to a device accumulator) and
// the arg-min over the candidates, so that a C caller can run the whole search without host arithmetic.
#include <mutex>

#include "svdq_dev.h"
#include "svdq_kernels.h"

namespace svdq {

namespace {

// Partial sums of svdq_sq_error_static: one file-scope array per GPU (each device that loads the library holds its
// own copy until the process ends), for callers that may not allocate.  In host code this name is only a handle:
// the device address comes from hipGetSymbolAddress (static_partials below) and is what the kernels receive.
static __device__ __align__(256) double scratch[SQ_ERROR_PARTIALS];

__global__ __launch_bounds__(256)
void sq_error_partial_kernel(const uint16_t* __restrict__ yref, int64_t ldr, const uint16_t* __restrict__ y, int64_t ldy,
                             int64_t M, int N, double* __restrict__ partials) {
    __shared__ double red[256];
    const int64_t chunks_per_row = N >> 3;                    // N % 8 == 0
    const int64_t total = M * chunks_per_row;
    double acc = 0.0;
    for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < total; c += (int64_t)gridDim.x * 256) {
        const int64_t m = c / chunks_per_row, n = (c - m * chunks_per_row) << 3;
        const uint4 a = *reinterpret_cast<const uint4*>(yref + m * ldr + n);
        const uint4 b = *reinterpret_cast<const uint4*>(y + m * ldy + n);
        const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
        float s = 0.0f;                                       // 8 squared differences: binary32 is ample
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float d0 = bf16lo_f(aw[i]) - bf16lo_f(bw[i]);
            const float d1 = bf16hi_f(aw[i]) - bf16hi_f(bw[i]);
            s = __builtin_fmaf(d0, d0, s);
            s = __builtin_fmaf(d1, d1, s);
        }
        acc += (double)s;
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) partials[blockIdx.x] = red[0];
}

// ADD = true: out[0] += the sum (one thread, so the accumulation over calls on a stream is deterministic)
template <bool ADD>
__global__ void sq_error_final_kernel(const double* __restrict__ partials, int n, double* __restrict__ out) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        double s = 0.0;
        for (int i = 0; i < n; ++i) s += partials[i];
        out[0] = ADD ? out[0] + s : s;
    }
}

// idx[row] = first index of the smallest entry of table[row][0..ncols): one thread per row
__global__ void argmin_rows_kernel(const double* __restrict__ table, int nrows, int ncols, int32_t* __restrict__ idx) {
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= nrows) return;
    const double* t = table + (size_t)row * ncols;
    int best = 0;
    for (int c = 1; c < ncols; ++c)
        if (t[c] < t[best]) best = c;
    idx[row] = best;
}

// Device address of `scratch` on the current device, looked up once per device.
hipError_t static_partials(double** out) {
    static std::mutex mu;
    static double* ptr[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        double* p = nullptr;
        e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return hipSuccess;
}

}  // namespace

hipError_t launch_sq_error(const void* yref, int64_t ldr, const void* y, int64_t ldy, int64_t M, int N,
                           double* workspace, double* out, bool add, hipStream_t stream) {
    hipLaunchKernelGGL(sq_error_partial_kernel, dim3(SQ_ERROR_PARTIALS), dim3(256), 0, stream,
                       (const uint16_t*)yref, ldr, (const uint16_t*)y, ldy, M, N, workspace);
    if (add)
        hipLaunchKernelGGL(sq_error_final_kernel<true>, dim3(1), dim3(64), 0, stream, workspace, SQ_ERROR_PARTIALS, out);
    else
        hipLaunchKernelGGL(sq_error_final_kernel<false>, dim3(1), dim3(64), 0, stream, workspace, SQ_ERROR_PARTIALS, out);
    return hipGetLastError();
}

// The same two kernels with the partial sums in this GPU's `scratch`: no allocation, no workspace argument.  Every
// block writes its partial sum on every call, so nothing has to be cleared between calls.
hipError_t launch_sq_error_static(const void* yref, int64_t ldr, const void* y, int64_t ldy, int64_t M, int N,
                                  double* out, hipStream_t stream) {
    double* partials = nullptr;
    const hipError_t e = static_partials(&partials);
    if (e != hipSuccess) return e;
    return launch_sq_error(yref, ldr, y, ldy, M, N, partials, out, false, stream);
}

hipError_t launch_argmin_rows(const double* table, int nrows, int ncols, int32_t* idx, hipStream_t stream) {
    hipLaunchKernelGGL(argmin_rows_kernel, dim3((unsigned)((nrows + 63) / 64)), dim3(64), 0, stream, table, nrows, ncols, idx);
    return hipGetLastError();
}

}  // namespace svdq
