// Kernels (b)+(c): W4A4 GEMM on the int8 matrix cores with one int32
// accumulator per 64-group, binary32 dequantisation, and the fused epilogue
// y = main + h L2 + bias (eq. 7 / eq. 11).
//
// The fp32 dequant step y += acc * sx[m,g] * sw[g,n] is what bounds this kernel:
// per 32x32 tile and group the int8 matrix core needs 64 clocks, while two FMAs
// per output on the (non-packed) vector ALU need 128.  So the work is moved:
//
//  * int4 -> int8 without sign extension.  `v & 0xF0F0F0F0` leaves the odd codes
//    of a packed dword as 16*q per byte, `(v << 4) & 0xF0F0F0F0` the even ones.
//    Both operands are scaled by 16 and the K order inside a group is permuted
//    identically on both sides, so the MFMA returns 256 * sum q_x q_w.
//  * int32 -> binary32 for free.  The first MFMA of a group starts from the bit
//    pattern of 2.25f.  256*acc fits in the mantissa below and above it, so the
//    int32 result read as a float IS f = 2.25 + acc * 2^-14, exactly.
//  * the scale product S[n][m] = (sx[m,g] * 2^14) * sw[g,n] of a tile is an outer
//    product, i.e. a matrix product with K = 1: the bf16 matrix core forms it
//    from hi+lo bf16 pieces of both scales (4 products, 16 significant bits).
//    The vector ALU is left with ONE FMA per output and group: y += f * S.
//  * that FMA also adds 2.25 * S.  Every second group a bf16 MFMA subtracts
//    2.25 * (S_g + S_{g+1}) straight into y (2.25 = 2 + 1/4, both exact factors
//    on bf16 pieces, same four products as S), so y never drifts far from the
//    true partial sum.
//
// Orientation: the MFMA computes the transposed tile D[n][m] (weights are the A
// operand).  Everything the matrix cores consume reaches them through LDS, staged
// one stage (two groups) ahead by the whole block, so the compute path has no
// global-memory waits: activations are unpacked to 16*q bytes while being staged;
// weights stay 4-bit in LDS (prepacked offline in fragment order) and are unpacked
// in registers; the bf16 pieces of the weight scales and the correction operands
// are prepacked offline too.  Block tile 128 x 128, 4 waves of 64 x 64.
#include "svdq_dev.h"
#include "svdq_kernels.h"

namespace svdq {

namespace {

constexpr int BM = 128, BN = 128;
constexpr int GS = 2;                          // groups per LDS stage
constexpr int LDS_ROW = 80;                    // 64 operand bytes + 16 pad: conflict-free 16-byte reads
constexpr uint32_t MAGIC_BITS = 0x40100000u;   // 2.25f
constexpr float SX_SCALE = 16384.0f;           // 2^14 = 2^22 / 256

struct Stage {
    uint8_t a[GS][BM * LDS_ROW];               // activations, 16*q per byte, chunk = 2*(odd codes) + 16-byte half
    uint4 w[GS][BN / 32][64];                  // weight fragments, still 4-bit: [group][n-block][lane]
    uint2 sxs[GS][BM];                         // {p, p}: m-side operand of the scale-product MFMA (K = 8), p = bf16 hi | lo << 16 of sx*2^14
    uint2 sfr[GS][BN / 32][32];                // n-side operand of the scale-product MFMA: bf16 {w1, w1, w2, w2}
    uint4 cfr[BN / 32][64];                    // n-side operand of the correction MFMA for this pair of groups
};

__device__ __forceinline__ void unpack_store(uint8_t* dst_row, int sp, uint4 v) {
    uint4 lo, hi;
    lo.x = (v.x << 4) & 0xF0F0F0F0u; hi.x = v.x & 0xF0F0F0F0u;
    lo.y = (v.y << 4) & 0xF0F0F0F0u; hi.y = v.y & 0xF0F0F0F0u;
    lo.z = (v.z << 4) & 0xF0F0F0F0u; hi.z = v.z & 0xF0F0F0F0u;
    lo.w = (v.w << 4) & 0xF0F0F0F0u; hi.w = v.w & 0xF0F0F0F0u;
    *reinterpret_cast<uint4*>(dst_row + sp * 16) = lo;            // k-step 0: even codes
    *reinterpret_cast<uint4*>(dst_row + (2 + sp) * 16) = hi;      // k-step 1: odd codes
}

// hi | lo << 16 bf16 pieces of v (16 significant bits)
__device__ __forceinline__ uint32_t split_bf16(float v) {
    const uint32_t hi = f_bf16_rne(v);
    const uint32_t lo = f_bf16_rne(v - bits_f(hi << 16));
    return hi | (lo << 16);
}

// sizes of the packed weight regions (bytes)
__host__ __device__ inline size_t wfrag_bytes(int N, int K) { return (size_t)N * (K / 2); }
__host__ __device__ inline size_t sfrag_bytes(int N, int K) { return (size_t)(N / 32) * (K / 64) * 256; }
__host__ __device__ inline size_t cfrag_bytes(int N, int K) { return (size_t)(N / 32) * ((K / 64 + 1) / 2) * 1024; }

// DUMP = false: the layer.  DUMP = true: write the int32 group accumulators of
// rows [dm0, dm0 + dmt) instead of y.
template <bool DUMP>
__global__ __launch_bounds__(256, 2)
void gemm_kernel(const uint8_t* __restrict__ qx, const float* __restrict__ sx,
                 const uint4* __restrict__ wfrag, const uint2* __restrict__ sfrag, const uint4* __restrict__ cfrag,
                 const float* __restrict__ h, const uint16_t* __restrict__ L2, const float* __restrict__ bias,
                 int64_t M, int64_t ldm, int N, int K, int r, void* __restrict__ yout, int64_t ldy, int out_f32,
                 int mtiles, int ntiles, int64_t dm0, int dmt, int32_t* __restrict__ dacc) {
    __shared__ __attribute__((aligned(16))) Stage stage[2];
    __shared__ __attribute__((aligned(16))) uint2 zero_entry;

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
    const int ngp = (ng + 1) >> 1;
    const int nstages = ngp;
    const int64_t m0 = (int64_t)mt * BM;
    const int n0 = nt * BN;

    // ---- staging assignment.  Per stage (two groups) a thread moves: 2 x 16 B of activation codes,
    // 2 x 16 B of weight fragments, 8 B of weight-scale pieces, 16 B of correction operand, one sx.
    const int srow = tid >> 1, sp = tid & 1;
    const int64_t arow = (m0 + srow < M) ? (m0 + srow) : (M - 1);
    const uint8_t* ga = qx + arow * 32 + sp * 16;                 // group-major codes: qx[g][row][32 B]
    const int xrow = tid & 127, xg = tid >> 7;                     // sx: threads 0..127 first group, 128..255 second
    const int64_t sxrow = (m0 + xrow < M) ? (m0 + xrow) : (M - 1);
    const float* gsx = DUMP ? nullptr : sx + sxrow;               // group-major scales: sx[g][row]
    const int nbB = n0 >> 5;                                       // first 32-channel block of this tile
    const int wnb = tid >> 6;                                      // weight fragment: (n-block = tid / 64, lane = tid % 64)
    const uint4* gw = wfrag + ((size_t)(nbB + wnb) * ng) * 64 + lane;
    const int snb = (tid >> 5) & 3, sj = tid >> 7;                 // scale pieces: (group = tid / 128, n-block, lane % 32)
    const uint2* gs = DUMP ? nullptr : sfrag + ((size_t)(nbB + snb) * ng) * 32 + l32;
    const uint4* gc = DUMP ? nullptr : cfrag + ((size_t)(nbB + wnb) * ngp) * 64 + lane;

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
    // opaque to the compiler: otherwise it rebuilds these 16 registers from a scalar before every use
    asm volatile("" : "+v"(magic));
    float16v zero16;
#pragma unroll
    for (int i = 0; i < 16; ++i) zero16[i] = 0.0f;

    // Plain locals (not a struct): a struct passed around by reference is not split into registers and
    // ends up in LDS, with a wait for the loads right after they are issued.
#define SVDQ_STAGE_LOAD(s_)                                                                              \
    {                                                                                                    \
        const int ga_ = ((s_) * GS < ng) ? (s_) * GS : (ng - 1);                                         \
        const int gb_ = ((s_) * GS + 1 < ng) ? (s_) * GS + 1 : (ng - 1);   /* odd tail: re-read the last group */ \
        va0 = *reinterpret_cast<const uint4*>(ga + (size_t)ga_ * ldm * 32);                              \
        va1 = *reinterpret_cast<const uint4*>(ga + (size_t)gb_ * ldm * 32);                              \
        vw0 = gw[(size_t)ga_ * 64];                                                                      \
        vw1 = gw[(size_t)gb_ * 64];                                                                      \
        if (!DUMP) {                                                                                     \
            const int gsj_ = ((s_) * GS + sj < ng) ? (s_) * GS + sj : (ng - 1);                          \
            vs = gs[(size_t)gsj_ * 32];                                                                  \
            vc = gc[(size_t)(s_) * 64];                                                                  \
            const int gx_ = (s_) * GS + xg;                                                              \
            sc = gsx[(size_t)(gx_ < ng ? gx_ : ng - 1) * ldm];                                           \
            sc_live = gx_ < ng;        /* applied at store time: using sc here would wait for the load */ \
        }                                                                                                \
    }
#define SVDQ_STAGE_STORE(st_)                                                                            \
    {                                                                                                    \
        unpack_store((st_).a[0] + srow * LDS_ROW, sp, va0);                                              \
        unpack_store((st_).a[1] + srow * LDS_ROW, sp, va1);                                              \
        (st_).w[0][wnb][lane] = vw0;                                                                     \
        (st_).w[1][wnb][lane] = vw1;                                                                     \
        if (!DUMP) {                                                                                     \
            (st_).sfr[sj][snb][l32] = vs;                                                                \
            (st_).cfr[wnb][lane] = vc;                                                                   \
            const uint32_t p_ = sc_live ? split_bf16(sc * SX_SCALE) : 0u;                                             \
            (st_).sxs[xg][xrow] = uint2{p_, p_};                                                         \
        }                                                                                                \
    }
    uint4 va0, va1, vw0, vw1, vc = {0u, 0u, 0u, 0u};
    uint2 vs = {0u, 0u};
    float sc = 0.0f;
    bool sc_live = false;

    // prologue: stage 0
    SVDQ_STAGE_LOAD(0);
    SVDQ_STAGE_STORE(stage[0]);
    if (tid == 0) zero_entry = uint2{0u, 0u};
    __syncthreads();

    for (int s = 0; s < nstages; ++s) {
        const Stage& cur = stage[s & 1];
        Stage& nxt = stage[(s + 1) & 1];
        const bool more = (s + 1 < nstages);
        if (more) SVDQ_STAGE_LOAD(s + 1);

#pragma unroll
        for (int j = 0; j < GS; ++j) {
            const int g = s * GS + j;
            if (g >= ng) break;

            // every LDS operand of this group is requested up front (and the scheduler may not sink the
            // reads next to their uses): LDS latency is then paid once per group, not once per MFMA
            int4v xf[2][2];
            uint2 sxs[2], sfr[2];
            uint4 wpk[2], cn[2];
            uint32_t cp_[2];
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                const int rrow = wm * 64 + mi * 32 + l32;
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
                    xf[mi][ks] = *reinterpret_cast<const int4v*>(cur.a[j] + rrow * LDS_ROW + (2 * ks + kh) * 16);
                if (!DUMP) {
                    const uint2* pe = kh ? &zero_entry : &cur.sxs[j][rrow];
                    sxs[mi] = *pe;
                    if (j == 0) cp_[mi] = cur.sxs[kh][rrow].x;     // lanes 0..31: group g, lanes 32..63: group g+1
                }
            }
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                wpk[ni] = cur.w[j][wn * 2 + ni][lane];
                if (!DUMP) {
                    const uint2* pe = kh ? &zero_entry : &cur.sfr[j][wn * 2 + ni][l32];
                    sfr[ni] = *pe;
                    if (j == 0) cn[ni] = cur.cfr[wn * 2 + ni][lane];
                }
            }
            __builtin_amdgcn_sched_barrier(0);

            if (!DUMP && j == 0) {
                // y -= 2.25 * (S_g + S_{g+1}) for the four tiles, before the two groups add it back
#pragma unroll
                for (int mi = 0; mi < 2; ++mi) {
                    const uint4 cm = {cp_[mi], cp_[mi], cp_[mi], cp_[mi]};
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni)
                        y[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, cn[ni]),
                                                                            __builtin_bit_cast(bf16x8, cm), y[ni][mi], 0, 0, 0);
                }
            }

#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                // int4 -> 16*q bytes, in registers (this wave's 32 output channels)
                int4v wlo, whi;
                const uint32_t pk[4] = {wpk[ni].x, wpk[ni].y, wpk[ni].z, wpk[ni].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    wlo[e] = (int)((pk[e] << 4) & 0xF0F0F0F0u);
                    whi[e] = (int)(pk[e] & 0xF0F0F0F0u);
                }
#pragma unroll
                for (int mi = 0; mi < 2; ++mi) {
                    int16v acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wlo, xf[mi][0], magic, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(whi, xf[mi][1], acc, 0, 0, 0);
                    if (DUMP) {
                        const int64_t m = m0 + wm * 64 + mi * 32 + l32;
                        if (m >= dm0 && m < dm0 + dmt && m < M) {
#pragma unroll
                            for (int i = 0; i < 16; ++i) {
                                const int n = n0 + wn * 64 + ni * 32 + 8 * (i >> 2) + 4 * kh + (i & 3);
                                dacc[((m - dm0) * N + n) * ng + g] = (acc[i] - (int)MAGIC_BITS) >> 8;
                            }
                        }
                    } else {
                        const float16v S = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(__builtin_bit_cast(short4v, sfr[ni]),
                                                                                    __builtin_bit_cast(short4v, sxs[mi]), zero16, 0, 0, 0);
#pragma unroll
                        for (int i = 0; i < 16; ++i)
                            y[ni][mi][i] = __builtin_fmaf(bits_f((uint32_t)acc[i]), S[i], y[ni][mi][i]);
                    }
                }
            }
        }

        if (more) SVDQ_STAGE_STORE(nxt);
        __syncthreads();
    }

#undef SVDQ_STAGE_LOAD
#undef SVDQ_STAGE_STORE
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

// Offline packing.  Region 1: weight fragments [N/32][K/64][64 lanes][16 B]: lane (n = lane % 32, kh = lane / 32)
// holds bytes [32 g + 16 kh, +16) of row n of the canonical codes.  Region 2: n-side operands of the
// scale-product MFMA, same indexing: lanes kh = 0 hold bf16 {w1, w1, w2, w2, 0, 0, 0, 0} with w1 + w2 ~ sw[g][n],
// lanes kh = 1 zeros.  Region 3: n-side operands of the correction MFMA [N/32][ceil(ng/2)][64][16 B]: lane
// (n, kh) holds, for group 2 gp + kh, bf16 {-2 w1, -2 w1, -2 w2, -2 w2, -w1/4, -w1/4, -w2/4, -w2/4}.
__global__ void pack_weight_kernel(const uint8_t* __restrict__ qw, const float* __restrict__ sw,
                                   int N, int K, uint8_t* __restrict__ out) {
    const int ng = K >> 6, ngp = (ng + 1) >> 1;
    const size_t stride = (size_t)gridDim.x * blockDim.x, t0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint4* o1 = reinterpret_cast<uint4*>(out);
    const size_t n1 = (size_t)(N >> 5) * ng * 64;
    for (size_t v = t0; v < n1; v += stride) {
        const int lane = (int)(v & 63);
        const size_t fr = v >> 6;
        const int g = (int)(fr % ng), nb = (int)(fr / ng);
        const int n = nb * 32 + (lane & 31), kh = lane >> 5;
        o1[v] = *reinterpret_cast<const uint4*>(qw + (size_t)n * (K >> 1) + g * 32 + kh * 16);
    }
    uint2* o2 = reinterpret_cast<uint2*>(out + wfrag_bytes(N, K));
    const size_t n2 = (size_t)(N >> 5) * ng * 32;
    for (size_t v = t0; v < n2; v += stride) {
        const int l = (int)(v & 31);
        const size_t fr = v >> 5;
        const int g = (int)(fr % ng), nb = (int)(fr / ng);
        const uint32_t p = split_bf16(sw[(size_t)g * N + nb * 32 + l]);
        const uint32_t w1 = p & 0xffffu, w2 = p >> 16;
        o2[v] = uint2{w1 | (w1 << 16), w2 | (w2 << 16)};
    }
    uint4* o3 = reinterpret_cast<uint4*>(out + wfrag_bytes(N, K) + sfrag_bytes(N, K));
    const size_t n3 = (size_t)(N >> 5) * ngp * 64;
    for (size_t v = t0; v < n3; v += stride) {
        const int lane = (int)(v & 63);
        const size_t fr = v >> 6;
        const int gp = (int)(fr % ngp), nb = (int)(fr / ngp);
        const int n = nb * 32 + (lane & 31), g = 2 * gp + (lane >> 5);
        uint4 e = {0u, 0u, 0u, 0u};
        if (g < ng) {
            const uint32_t p = split_bf16(sw[(size_t)g * N + n]);
            const float w1 = bits_f(p << 16), w2 = bits_f(p & 0xffff0000u);
            // exact: powers of two times bf16 values (barring underflow)
            const uint32_t a1 = f_bf16_rne(-2.0f * w1), a2 = f_bf16_rne(-2.0f * w2);
            const uint32_t b1 = f_bf16_rne(-0.25f * w1), b2 = f_bf16_rne(-0.25f * w2);
            e.x = a1 | (a1 << 16);
            e.y = a2 | (a2 << 16);
            e.z = b1 | (b1 << 16);
            e.w = b2 | (b2 << 16);
        }
        o3[v] = e;
    }
}

}  // namespace

size_t packed_weight_bytes(int N, int K) { return wfrag_bytes(N, K) + sfrag_bytes(N, K) + cfrag_bytes(N, K); }

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
    const uint8_t* base = (const uint8_t*)w_packed;
    const uint4* wf = (const uint4*)base;
    const uint2* sf = (const uint2*)(base + wfrag_bytes(N, K));
    const uint4* cf = (const uint4*)(base + wfrag_bytes(N, K) + sfrag_bytes(N, K));
    hipLaunchKernelGGL(gemm_kernel<false>, dim3(grid_for(mtiles, ntiles)), dim3(256), 0, stream,
                       qx, sx, wf, sf, cf, h, (const uint16_t*)L2, bias, M, M, N, K, r, y, ldy, out_f32,
                       mtiles, ntiles, (int64_t)0, 0, (int32_t*)nullptr);
    return hipGetLastError();
}

hipError_t launch_group_acc(const uint8_t* qx, const void* w_packed, int64_t M, int N, int K,
                            int64_t m0, int mt, int32_t* acc, hipStream_t stream) {
    // only the token tiles that intersect [m0, m0 + mt) are launched
    const int t0 = (int)(m0 / BM), t1 = (int)((m0 + mt + BM - 1) / BM);
    const int mtiles = t1 - t0, ntiles = N / BN;
    const int64_t off = (int64_t)t0 * BM;
    // the integer accumulators need no scales: the DUMP instantiation never reads them
    hipLaunchKernelGGL(gemm_kernel<true>, dim3(grid_for(mtiles, ntiles)), dim3(256), 0, stream,
                       qx + off * 32, (const float*)nullptr, (const uint4*)w_packed, (const uint2*)nullptr,
                       (const uint4*)nullptr, (const float*)nullptr, (const uint16_t*)nullptr,
                       (const float*)nullptr, M - off, M, N, K, 0, (void*)nullptr, (int64_t)0, 0,
                       mtiles, ntiles, m0 - off, mt, acc);
    return hipGetLastError();
}

}  // namespace svdq
