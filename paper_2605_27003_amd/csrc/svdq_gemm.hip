// Kernels (b)+(c): W4A4 GEMM on the int8 matrix cores with one int32
// accumulator per 64-group, binary32 dequantisation, and the fused epilogue
// y = main + h L2 + bias (eq. 7 / eq. 11).
//
// Block tile 128 (tokens) x 128 (output channels), 4 waves of 64 x 64, one
// 64-group per main-loop step, two LDS stages.
//
// int4 -> int8 without sign extension.  A packed dword holds 8 nibbles; `v &
// 0xF0F0F0F0` leaves the odd codes as 16*q in each byte and `(v << 4) &
// 0xF0F0F0F0` does the same for the even codes.  Both operands are scaled by
// 16, the K order inside a group is permuted identically for activations and
// weights (an integer dot product does not care), so the matrix core returns
// 256 * sum q_x q_w.  The unpack happens once per block when a tile is staged
// into LDS, not per wave.
//
// int32 -> binary32 for free.  The first MFMA of a group starts from the bit
// pattern of 3.0f instead of 0.  256*acc fits in the mantissa below it, so the
// int32 result, read as a float, IS 3 + acc * 2^-14, exactly.  The dequant
// step is then two FMAs per output and group:
//     t = f * (sx * 2^14) + (-3 * sx * 2^14)      ( = acc * sx )
//     y = t * sw + y
// Orientation: the MFMA computes the transposed tile D[n][m], so a lane owns
// one token m (its sx terms are per-lane scalars) and 16 output channels n.
#include "svdq_dev.h"
#include "svdq_kernels.h"

namespace svdq {

namespace {

constexpr int BM = 128, BN = 128;
constexpr int LDS_ROW = 80;                 // 64 operand bytes + 16 pad: conflict-free 16-byte reads
constexpr uint32_t MAGIC_BITS = 0x40400000u;   // 3.0f
constexpr float SX_SCALE = 16384.0f;        // 2^14 = 2^22 / 256

struct Stage {
    uint8_t a[BM * LDS_ROW];                // activations, 16*q per byte
    uint8_t w[BN * LDS_ROW];                // weights, 16*q per byte
    float sr[BM];                           // sx * 2^14
    float sw[BN];
};

__device__ __forceinline__ void unpack_store(uint8_t* dst_row, int p, uint4 v) {
    uint4 lo, hi;
    lo.x = (v.x << 4) & 0xF0F0F0F0u; hi.x = v.x & 0xF0F0F0F0u;
    lo.y = (v.y << 4) & 0xF0F0F0F0u; hi.y = v.y & 0xF0F0F0F0u;
    lo.z = (v.z << 4) & 0xF0F0F0F0u; hi.z = v.z & 0xF0F0F0F0u;
    lo.w = (v.w << 4) & 0xF0F0F0F0u; hi.w = v.w & 0xF0F0F0F0u;
    *reinterpret_cast<uint4*>(dst_row + (2 * p) * 16) = lo;
    *reinterpret_cast<uint4*>(dst_row + (2 * p + 1) * 16) = hi;
}

// DUMP = false: the layer.  DUMP = true: write the int32 group accumulators of
// rows [dm0, dm0 + dmt) instead of y.
template <bool DUMP>
__global__ __launch_bounds__(256, 2)
void gemm_kernel(const uint8_t* __restrict__ qx, const float* __restrict__ sx,
                 const uint8_t* __restrict__ wq, const float* __restrict__ sw,
                 const float* __restrict__ h, const uint16_t* __restrict__ L2, const float* __restrict__ bias,
                 int64_t M, int N, int K, int r, void* __restrict__ yout, int64_t ldy, int out_f32,
                 int mtiles, int ntiles, int64_t dm0, int dmt, int32_t* __restrict__ dacc) {
    __shared__ __attribute__((aligned(16))) Stage stage[2];

    // XCD-aware tile order: consecutive block ids go round-robin to the 8 XCDs,
    // so give each XCD its own token tiles and walk them 8 at a time across n.
    const int bid = blockIdx.x;
    const int xcd = bid & 7, idx = bid >> 3;
    const int sm = idx / (8 * ntiles), rem = idx - sm * (8 * ntiles);
    const int nt = rem >> 3;
    const int mt = (sm * 8 + (rem & 7)) * 8 + xcd;
    if (mt >= mtiles) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int l32 = lane & 31, kh = lane >> 5;
    const int ng = K >> 6;
    const int64_t m0 = (int64_t)mt * BM;
    const int n0 = nt * BN;

    // staging assignment: thread -> (row, 16-byte half of the group's 32 packed bytes)
    const int srow = tid >> 1, sp = tid & 1;
    const int64_t arow = (m0 + srow < M) ? (m0 + srow) : (M - 1);
    const uint8_t* ga = qx + arow * (int64_t)(K >> 1) + sp * 16;
    const uint8_t* gw = wq + ((size_t)nt * ng * BN + srow) * 32 + sp * 16;
    // scale staging: threads 0..127 fetch sw, 128..255 fetch sx
    const int64_t sxrow = (m0 + (tid & 127) < M) ? (m0 + (tid & 127)) : (M - 1);
    const float* gs = DUMP ? nullptr : ((tid < 128) ? (sw + n0 + tid) : (sx + sxrow * ng));
    const int64_t gs_step = (tid < 128) ? N : 1;

    float16v y[2][2];                        // [ni][mi]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) y[a][b][i] = 0.0f;

    int16v magic;
#pragma unroll
    for (int i = 0; i < 16; ++i) magic[i] = (int)MAGIC_BITS;

    // prologue: group 0 -> stage 0
    {
        uint4 va = *reinterpret_cast<const uint4*>(ga);
        uint4 vw = *reinterpret_cast<const uint4*>(gw);
        float sc = DUMP ? 1.0f : gs[0];
        unpack_store(stage[0].a + srow * LDS_ROW, sp, va);
        unpack_store(stage[0].w + srow * LDS_ROW, sp, vw);
        if (tid < 128) stage[0].sw[tid] = sc; else stage[0].sr[tid - 128] = sc * SX_SCALE;
    }
    __syncthreads();

    for (int g = 0; g < ng; ++g) {
        const Stage& cur = stage[g & 1];
        Stage& nxt = stage[(g + 1) & 1];
        const bool more = (g + 1 < ng);
        uint4 va, vw;
        float sc = 0.0f;
        if (more) {
            va = *reinterpret_cast<const uint4*>(ga + (size_t)(g + 1) * 32);
            vw = *reinterpret_cast<const uint4*>(gw + (size_t)(g + 1) * BN * 32);
            if (!DUMP) sc = gs[(int64_t)(g + 1) * gs_step];
        }

        // per-lane token scales and per-register channel scales of this group
        float srv[2], crv[2];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
            srv[mi] = cur.sr[wm * 64 + mi * 32 + l32];
            crv[mi] = -3.0f * srv[mi];
        }
        float swv[2][16];
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float4 t = *reinterpret_cast<const float4*>(&cur.sw[wn * 64 + ni * 32 + 8 * q + 4 * kh]);
                swv[ni][4 * q + 0] = t.x; swv[ni][4 * q + 1] = t.y; swv[ni][4 * q + 2] = t.z; swv[ni][4 * q + 3] = t.w;
            }

        int16v acc[2][2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            int4v wf[2], xf[2];
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
                wf[ni] = *reinterpret_cast<const int4v*>(cur.w + (wn * 64 + ni * 32 + l32) * LDS_ROW + (2 * ks + kh) * 16);
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
                xf[mi] = *reinterpret_cast<const int4v*>(cur.a + (wm * 64 + mi * 32 + l32) * LDS_ROW + (2 * ks + kh) * 16);
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
                    acc[ni][mi] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[ni], xf[mi], ks == 0 ? magic : acc[ni][mi], 0, 0, 0);
        }

        if (DUMP) {
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int mi = 0; mi < 2; ++mi) {
                    int64_t m = m0 + wm * 64 + mi * 32 + l32;
                    if (m >= dm0 && m < dm0 + dmt && m < M) {
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            int n = n0 + wn * 64 + ni * 32 + 8 * (i >> 2) + 4 * kh + (i & 3);
                            dacc[((m - dm0) * N + n) * ng + g] = (acc[ni][mi][i] - (int)MAGIC_BITS) >> 8;
                        }
                    }
                }
        } else {
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        float t = __builtin_fmaf(bits_f((uint32_t)acc[ni][mi][i]), srv[mi], crv[mi]);
                        y[ni][mi][i] = __builtin_fmaf(t, swv[ni][i], y[ni][mi][i]);
                    }
        }

        if (more) {
            unpack_store(nxt.a + srow * LDS_ROW, sp, va);
            unpack_store(nxt.w + srow * LDS_ROW, sp, vw);
            if (tid < 128) nxt.sw[tid] = sc; else nxt.sr[tid - 128] = sc * SX_SCALE;
        }
        __syncthreads();
    }

    if (DUMP) return;

    // ---- epilogue (c): low-rank up-projection on the bf16 matrix cores, bias, store
    if (r > 0) {
        const int ksteps = r >> 4;
        for (int ks = 0; ks < ksteps; ++ks) {
            bf16x8 lf[2];                      // L2^T fragment: row n, k = j
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                const int n = n0 + wn * 64 + ni * 32 + l32;
                uint32_t wds[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    uint32_t lo = L2[(int64_t)(16 * ks + 8 * kh + 2 * e) * N + n];
                    uint32_t hi = L2[(int64_t)(16 * ks + 8 * kh + 2 * e + 1) * N + n];
                    wds[e] = lo | (hi << 16);
                }
                uint4 t = {wds[0], wds[1], wds[2], wds[3]};
                lf[ni] = __builtin_bit_cast(bf16x8, t);
            }
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                int64_t m = m0 + wm * 64 + mi * 32 + l32;
                if (m >= M) m = M - 1;
                const float4* ph = reinterpret_cast<const float4*>(h + m * r + 16 * ks + 8 * kh);
                float4 h0 = ph[0], h1 = ph[1];
                const float hv[8] = {h0.x, h0.y, h0.z, h0.w, h1.x, h1.y, h1.z, h1.w};
                uint32_t hi16[8], lo16[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    hi16[e] = f_bf16_rne(hv[e]);
                    lo16[e] = f_bf16_rne(hv[e] - bits_f(hi16[e] << 16));
                }
                uint4 th = {hi16[0] | (hi16[1] << 16), hi16[2] | (hi16[3] << 16), hi16[4] | (hi16[5] << 16), hi16[6] | (hi16[7] << 16)};
                uint4 tl = {lo16[0] | (lo16[1] << 16), lo16[2] | (lo16[3] << 16), lo16[4] | (lo16[5] << 16), lo16[6] | (lo16[7] << 16)};
                bf16x8 hhi = __builtin_bit_cast(bf16x8, th), hlo = __builtin_bit_cast(bf16x8, tl);
#pragma unroll
                for (int ni = 0; ni < 2; ++ni) {
                    y[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lf[ni], hhi, y[ni][mi], 0, 0, 0);
                    y[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lf[ni], hlo, y[ni][mi], 0, 0, 0);
                }
            }
        }
    }

#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int n = n0 + wn * 64 + ni * 32 + 8 * q + 4 * kh;
            float4 bv = {0.f, 0.f, 0.f, 0.f};
            if (bias) bv = *reinterpret_cast<const float4*>(bias + n);
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                const int64_t m = m0 + wm * 64 + mi * 32 + l32;
                if (m >= M) continue;
                float v0 = y[ni][mi][4 * q + 0] + bv.x, v1 = y[ni][mi][4 * q + 1] + bv.y;
                float v2 = y[ni][mi][4 * q + 2] + bv.z, v3 = y[ni][mi][4 * q + 3] + bv.w;
                if (out_f32) {
                    float4 o = {v0, v1, v2, v3};
                    *reinterpret_cast<float4*>(reinterpret_cast<float*>(yout) + m * ldy + n) = o;
                } else {
                    uint2 o = {f_bf16_rne(v0) | (f_bf16_rne(v1) << 16), f_bf16_rne(v2) | (f_bf16_rne(v3) << 16)};
                    *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(yout) + m * ldy + n) = o;
                }
            }
        }
    }
}

// canonical [N, K/2] codes -> [N/128][K/64][128][32] tiles, then the scales [K/64, N]
__global__ void pack_weight_kernel(const uint8_t* __restrict__ qw, const float* __restrict__ sw,
                                   int N, int K, uint8_t* __restrict__ out) {
    const int ng = K >> 6;
    const size_t nvec = (size_t)N * (K >> 1) / 16;
    for (size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x; v < nvec; v += (size_t)gridDim.x * blockDim.x) {
        // destination vector index -> (nt, g, row, p)
        int p = (int)(v & 1);
        int row = (int)((v >> 1) & 127);
        size_t rest = v >> 8;
        int g = (int)(rest % ng);
        int nt = (int)(rest / ng);
        const uint4* src = reinterpret_cast<const uint4*>(qw + ((size_t)(nt * BN + row)) * (K >> 1) + g * 32 + p * 16);
        reinterpret_cast<uint4*>(out)[v] = *src;
    }
    float* so = reinterpret_cast<float*>(out + (size_t)N * (K >> 1));
    const size_t ns = (size_t)ng * N;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < ns; i += (size_t)gridDim.x * blockDim.x) so[i] = sw[i];
}

}  // namespace

size_t packed_weight_bytes(int N, int K) {
    return (size_t)N * (K / 2) + (size_t)(K / 64) * N * sizeof(float);
}

hipError_t launch_pack_weight(const uint8_t* qw, const float* sw, int N, int K, void* out, hipStream_t stream) {
    hipLaunchKernelGGL(pack_weight_kernel, dim3(1024), dim3(256), 0, stream, qw, sw, N, K, (uint8_t*)out);
    return hipGetLastError();
}

static inline unsigned grid_for(int mtiles, int ntiles) {
    const int sms = (mtiles + 63) / 64;          // super-stripes of 8 XCDs x 8 token tiles
    return (unsigned)(sms * 64 * ntiles);
}

hipError_t launch_linear(const uint8_t* qx, const float* sx, const void* w_packed,
                         const float* h, const void* L2, const float* bias,
                         int64_t M, int N, int K, int r, void* y, int64_t ldy, int out_f32,
                         hipStream_t stream) {
    const int mtiles = (int)((M + BM - 1) / BM), ntiles = N / BN;
    const uint8_t* wq = (const uint8_t*)w_packed;
    const float* sw = (const float*)(wq + (size_t)N * (K / 2));
    hipLaunchKernelGGL(gemm_kernel<false>, dim3(grid_for(mtiles, ntiles)), dim3(256), 0, stream,
                       qx, sx, wq, sw, h, (const uint16_t*)L2, bias, M, N, K, r, y, ldy, out_f32,
                       mtiles, ntiles, (int64_t)0, 0, (int32_t*)nullptr);
    return hipGetLastError();
}

hipError_t launch_group_acc(const uint8_t* qx, const void* w_packed, int64_t M, int N, int K,
                            int64_t m0, int mt, int32_t* acc, hipStream_t stream) {
    // only the token tiles that intersect [m0, m0 + mt) are launched
    const int t0 = (int)(m0 / BM), t1 = (int)((m0 + mt + BM - 1) / BM);
    const int mtiles = t1 - t0, ntiles = N / BN;
    const uint8_t* wq = (const uint8_t*)w_packed;
    const float* sw = (const float*)(wq + (size_t)N * (K / 2));
    const int64_t off = (int64_t)t0 * BM;
    // the integer accumulators need no scales: the DUMP instantiation never reads them
    hipLaunchKernelGGL(gemm_kernel<true>, dim3(grid_for(mtiles, ntiles)), dim3(256), 0, stream,
                       qx + off * (K / 2), (const float*)nullptr, wq, sw, (const float*)nullptr, (const uint16_t*)nullptr,
                       (const float*)nullptr, M - off, N, K, 0, (void*)nullptr, (int64_t)0, 0,
                       mtiles, ntiles, m0 - off, mt, acc);
    return hipGetLastError();
}

}  // namespace svdq
