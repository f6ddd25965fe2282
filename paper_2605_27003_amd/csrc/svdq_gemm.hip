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
// one stage (two groups) ahead, so the compute path has no global-memory waits.
// Staging uses the direct global->LDS loads of gfx950 (global_load_lds_dwordx4):
// no registers, no VALU work and no ds_write for the bulk data.  Codes of both
// operands stay 4-bit in LDS and are unpacked in registers by the wave that
// multiplies them; weight fragments, the bf16 pieces of the weight scales and the
// correction operands are prepacked offline in fragment order; activations arrive
// group-major from the quantise kernel, which is fragment order already.
// Block tile 128 x 128, 4 waves of 64 x 64.
#include "svdq_dev.h"
#include "svdq_kernels.h"

namespace svdq {

namespace {

constexpr int BM = 128, BN = 128;
constexpr int GS = 2;                          // groups per LDS stage
constexpr uint32_t MAGIC_BITS = 0x40100000u;   // 2.25f
constexpr float SX_SCALE = 16384.0f;           // 2^14 = 2^22 / 256

struct Stage {
    uint4 a[GS][2][BM];                        // activation codes, 4-bit: [group][16-byte half of the group's 32 B][token]
    uint4 w[GS][BN / 32][64];                  // weight fragments, 4-bit: [group][n-block][lane]
    uint4 cfr[BN / 32][64];                    // n-side operand of the correction MFMA for this pair of groups
    uint2 sfr[GS][BN / 32][32];                // n-side operand of the scale-product MFMA: bf16 {w1, w1, w2, w2}
    uint2 sxs[GS][BM];                         // {p, p}: m-side operand of the scale-product MFMA (K = 8), p = bf16 hi | lo << 16 of sx*2^14
};

// One wave-wide direct global->LDS load: lane l moves 16 bytes from its own global address to LDS byte
// offset lds_off + 16 l.  Written as inline asm so that the compiler does not treat every later LDS
// read as dependent on it; the issuing code waits (vmcnt) and barriers before anyone reads the data.
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_off) {
    lds_off = __builtin_amdgcn_readfirstlane(lds_off);            // wave-uniform by construction: goes to M0
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_off) : "memory");
}
__device__ __forceinline__ uint32_t lds_offset(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

// 4-bit codes -> 16*q bytes: even codes of each byte pair (k-step 0) and odd codes (k-step 1)
__device__ __forceinline__ void unpack16(const uint4 v, int4v& lo, int4v& hi) {
    const uint32_t pk[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        lo[e] = (int)((pk[e] << 4) & 0xF0F0F0F0u);
        hi[e] = (int)(pk[e] & 0xF0F0F0F0u);
    }
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
    __shared__ __attribute__((aligned(16))) Stage stage[3];         // ring: consume s, s+1 landed/landing, s+2 in flight
    __shared__ __attribute__((aligned(16))) uint2 zero_entry;

    // XCD-aware tile order: consecutive block ids go round-robin to the 8 XCDs,
    // so give each XCD its own token tiles and walk them 8 at a time across n.
    const int bid = blockIdx.x;
    const int xcd = bid & 7, idx = bid >> 3;
    const int sm = idx / (8 * ntiles), rem = idx - sm * (8 * ntiles);
    const int nt = rem >> 3;
    const int mt = (sm * 8 + (rem & 7)) * 8 + xcd;
    if (mt >= mtiles) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);    // scalar: everything derived from it stays in SGPRs
    const int wm = wave & 1, wn = wave >> 1;
    const int l32 = lane & 31, kh = lane >> 5;
    const int ng = K >> 6;
    const int ngp = (ng + 1) >> 1;
    const int nstages = ngp;
    const int64_t m0 = (int64_t)mt * BM;
    const int n0 = nt * BN;

    // ---- staging.  Per stage (two groups) the block moves 8 KB of activation codes, 8 KB of weight
    // fragments, 4 KB of correction operands and 2 KB of weight-scale pieces with direct global->LDS
    // loads (1 KB per wave instruction, 5-6 instructions per wave), and 256 token scales through registers.
    const int xrow = tid & 127, xg = tid >> 7;                     // sx: threads 0..127 first group, 128..255 second
    const int64_t sxrow = (m0 + xrow < M) ? (m0 + xrow) : (M - 1);
    const float* gsx = DUMP ? nullptr : sx + sxrow;               // group-major scales: sx[g][row]
    const int nbB = n0 >> 5;                                       // first 32-channel block of this tile
    // activation chunks of this wave: c = 2 wave + {0,1} -> (group j = c/4, half sp = (c/2)%2, 64-row half rh = c%2)
    const uint8_t* ga[2];
    int aj[2], asp[2], arh[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = 2 * wave + i;
        aj[i] = c >> 2; asp[i] = (c >> 1) & 1; arh[i] = c & 1;
        const int64_t row = m0 + arh[i] * 64 + lane;
        ga[i] = qx + ((row < M) ? row : (M - 1)) * 32 + asp[i] * 16;       // + g * ldm * 32 per group
    }
    // weight chunks of this wave: c = 2 wave + {0,1} -> (group j = c/4, n-block = c%4)
    const uint4* gw[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) gw[i] = wfrag + ((size_t)(nbB + ((2 * wave + i) & 3)) * ng) * 64 + lane;
    const uint4* gc = DUMP ? nullptr : cfrag + ((size_t)(nbB + wave) * ngp) * 64 + lane;           // n-block = wave
    // scale pieces: waves 0 and 1 take group j = wave; lane -> (n-block = lane/16, two entries 2(lane%16), +1)
    const uint2* gs = DUMP ? nullptr : sfrag + ((size_t)(nbB + (lane >> 4)) * ng) * 32 + 2 * (lane & 15);

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

    float sc = 0.0f;
    bool sc_live = false;
    const int ndma = DUMP ? 4 : (wave < 2 ? 6 : 5);                 // direct-to-LDS loads this wave issues per stage
    // scale of this thread's (group, token) of stage s: through a register, issued BEFORE the bulk loads
    auto scale_issue = [&](const int s) {
        if (!DUMP) {
            const int gx = s * GS + xg;
            sc = gsx[(size_t)(gx < ng ? gx : ng - 1) * ldm];
            sc_live = gx < ng;                   // applied at store time: using sc here would wait for the load
        }
    };
    auto stage_issue = [&](const int s, Stage& st) {
        const int gj[2] = {(s * GS < ng) ? s * GS : ng - 1, (s * GS + 1 < ng) ? s * GS + 1 : ng - 1};   // odd tail: re-read
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            dma16(ga[i] + (size_t)gj[aj[i]] * ldm * 32, lds_offset(&st.a[aj[i]][asp[i]][arh[i] * 64]));
            dma16(gw[i] + (size_t)gj[(2 * wave + i) >> 2] * 64, lds_offset(&st.w[(2 * wave + i) >> 2][(2 * wave + i) & 3][0]));
        }
        if (!DUMP) {
            dma16(gc + (size_t)s * 64, lds_offset(&st.cfr[wave][0]));
            if (wave < 2) dma16(gs + (size_t)gj[wave] * 32, lds_offset(&st.sfr[wave][0][0]));
        }
    };
    auto scale_store = [&](Stage& st) {
        if (!DUMP) {
            const uint32_t p = sc_live ? split_bf16(sc * SX_SCALE) : 0u;
            st.sxs[xg][xrow] = uint2{p, p};
        }
    };
    // wait until at most `n` of this wave's vector-memory loads are outstanding (they complete in order)
    auto wait_loads = [&](const int n) {
        if (n == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        else if (n == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else if (n == 5) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
    };

    // prologue: stage 0 completely, bulk loads of stage 1 in flight
    scale_issue(0);
    stage_issue(0, stage[0]);
    if (nstages > 1) stage_issue(1, stage[1]);
    wait_loads(nstages > 1 ? ndma : 0);
    scale_store(stage[0]);
    if (tid == 0) zero_entry = uint2{0u, 0u};
    __syncthreads();

    int cur_i = 0;                                                  // ring index of the stage being consumed
    for (int s = 0; s < nstages; ++s) {
        const int nxt_i = (cur_i == 2) ? 0 : cur_i + 1;
        const int nn_i = (nxt_i == 2) ? 0 : nxt_i + 1;
        const Stage& cur = stage[cur_i];
        Stage& nxt = stage[nxt_i];
        const bool more = (s + 1 < nstages), more2 = (s + 2 < nstages);
        // order matters: the token scale of stage s+1 first, then the bulk loads of stage s+2, so that the
        // wait at the end of this stage (everything but the last ndma loads) covers all of stage s+1
        if (more) scale_issue(s + 1);
        if (more2) stage_issue(s + 2, stage[nn_i]);

#pragma unroll
        for (int j = 0; j < GS; ++j) {
            const int g = s * GS + j;
            if (g >= ng) break;

            // every LDS operand of this group is requested up front (and the scheduler may not sink the
            // reads next to their uses): LDS latency is then paid once per group, not once per MFMA
            uint4 xpk[2], wpk[2], cn[2];
            uint2 sxs[2], sfr[2];
            uint32_t cp_[2];
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                const int rrow = wm * 64 + mi * 32 + l32;
                xpk[mi] = cur.a[j][kh][rrow];
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

            // int4 -> 16*q bytes, in registers
            int4v xlo[2], xhi[2];
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) unpack16(xpk[mi], xlo[mi], xhi[mi]);
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                int4v wlo, whi;
                unpack16(wpk[ni], wlo, whi);
#pragma unroll
                for (int mi = 0; mi < 2; ++mi) {
                    int16v acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wlo, xlo[mi], magic, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(whi, xhi[mi], acc, 0, 0, 0);
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
            if (!DUMP && j == 0) {
                // y -= 2.25 * (S_g + S_{g+1}) for the four tiles, between the two groups that add it: y then strays
                // from the true partial sum by at most 2.25 * S in either direction
#pragma unroll
                for (int mi = 0; mi < 2; ++mi) {
                    const uint4 cm = {cp_[mi], cp_[mi], cp_[mi], cp_[mi]};
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni)
                        y[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, cn[ni]),
                                                                            __builtin_bit_cast(bf16x8, cm), y[ni][mi], 0, 0, 0);
                }
            }

        }

        if (more) {
            wait_loads(more2 ? ndma : 0);
            scale_store(nxt);
        }
        __syncthreads();
        cur_i = nxt_i;
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
