// MXFP4 variant of the layer: the 4-bit format of the paper's Table I (E2M1 elements, one E8M0
// power-of-two scale per 32 values along K) on the block-scaled matrix instruction of gfx950,
// v_mfma_scale_f32_32x32x64_f8f6f4.  The matrix core applies both operands' block scales itself and
// accumulates in binary32 across all of K, so the per-group dequantisation that bounds the int4 kernel
// (one vector FMA per output and 64 of K) does not exist here: the K loop is matrix instructions and
// operand movement only.
//
// Operand layout of that instruction for 4-bit data (checked against a host reference with random
// codes and scales): lane l holds row (l % 32) of its operand and the 32 consecutive k
// [32 (l / 32), +32) as 16 bytes, code k in nibble (k % 8) of dword (k / 8) % 4; the scale register of
// lane l carries the E8M0 byte of exactly those 32 values (byte chosen by op_sel).  That is the
// group-major activation layout of the int4 path unchanged: 32 bytes per token and 64-group, a lane
// reads 16 of them.
//
// Kernel (a'): as the int4 quantise kernel (same lane layout, same low-rank down-projection on the
// bf16 matrix cores), but a lane's 32 values ARE one MX block: absmax needs no cross-lane step, the
// shared exponent is read off the binary32 exponent of rho * absmax (eq. 8), and
// v_cvt_scalef32_pk_fp4_f32 rounds two values at a time to E2M1 (nearest, ties to the even code,
// saturating; checked against the definition on 2e5 random and all boundary inputs).
#include <atomic>

#include "svdq_act.h"
#include "svdq_dev.h"
#include "svdq_epilogue.h"
#include "svdq_kernels.h"
#include "svdq_lds.h"
#include "svdq_tiles.h"

namespace svdq {

namespace {

typedef int int8v __attribute__((ext_vector_type(8)));

// ------------------------------------------------------------------------------------------------
// kernel (a'): smooth, per-token per-32-block shared exponent, E2M1 codes, h = x^ L1
// ------------------------------------------------------------------------------------------------
constexpr int QROWS = 64;     // token rows per block
constexpr int QWAVES = 4;     // K is split between the waves by stage (two 64-groups = 128 k)
constexpr int QHPART_BYTES = QWAVES * QROWS * 33 * 4;

// One 32-row block of one group: this lane's 32 values -> 16 bytes of codes and the block's E8M0 byte.
__device__ __forceinline__ void quantize_block_mx(const uint4 (&xv)[4], const float* __restrict__ il_lds, float rho,
                                                  uint4& codes, uint32_t& e8) {
    float xs[32];
    float a = 0.0f;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const float4 i0 = *reinterpret_cast<const float4*>(il_lds + 8 * s);
        const float4 i1 = *reinterpret_cast<const float4*>(il_lds + 8 * s + 4);
        const float ilv[8] = {i0.x, i0.y, i0.z, i0.w, i1.x, i1.y, i1.z, i1.w};
        const uint32_t wds[4] = {xv[s].x, xv[s].y, xv[s].z, xv[s].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float lo = __fmul_rn(bf16lo_f(wds[j]), ilv[2 * j]);          // eq. 5 in binary32
            float hi = __fmul_rn(bf16hi_f(wds[j]), ilv[2 * j + 1]);
            xs[8 * s + 2 * j] = lo;
            xs[8 * s + 2 * j + 1] = hi;
            a = __builtin_fmaxf(a, __builtin_fmaxf(__builtin_fabsf(lo), __builtin_fabsf(hi)));
        }
    }
    // eq. 8: alpha = rho * a is the block's reference magnitude; shared exponent floor(log2 alpha) - 2.
    // For a normal alpha the binary32 exponent field is floor(log2 alpha) + 127, so the E8M0 byte is that
    // field minus 2; below 2^-124 (field < 3) the block is empty.
    const uint32_t field = (f_bits(__fmul_rn(rho, a)) >> 23) & 0xffu;
    const bool live = field >= 3u;
    e8 = live ? field - 2u : 0u;
    const float X = bits_f((live ? field - 2u : 127u) << 23);           // 2^(byte - 127), a normal number
    uint32_t packed[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        uint32_t wd = 0;
        wd = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(wd, xs[8 * d + 0], xs[8 * d + 1], X, 0);
        wd = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(wd, xs[8 * d + 2], xs[8 * d + 3], X, 1);
        wd = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(wd, xs[8 * d + 4], xs[8 * d + 5], X, 2);
        wd = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(wd, xs[8 * d + 6], xs[8 * d + 7], X, 3);
        packed[d] = live ? wd : 0u;
    }
    codes = uint4{packed[0], packed[1], packed[2], packed[3]};
}

// Outputs: qx [K/64][M][32 B] (as the int4 path) and sxe [ceil(K/128)][M][2][2] bytes: for token m and stage s
// (groups 2s, 2s+1) the two bytes [half h][group j] are the E8M0 scales of MX block 2 (2s + j) + h.
// GELU = true: every x is replaced by bf16(gelu(x)) as it arrives (svdq_act.h).
template <bool LOWRANK, bool GELU>
__global__ __launch_bounds__(256, 2)
void quantize_mx_kernel(const uint16_t* __restrict__ x, int64_t ldx,
                        const float* __restrict__ inv_lambda, float rho,
                        const uint4* __restrict__ l1p, int64_t M, int K, int r,
                        uint8_t* __restrict__ qx, uint16_t* __restrict__ sxe, float* __restrict__ h) {
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    float* il_s = reinterpret_cast<float*>(smem_raw);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int rr = lane & 31;
    const int hf = lane >> 5;
    const int ng = K >> 6;
    const int nstages = (ng + 1) >> 1;
    const int64_t row0 = (int64_t)blockIdx.x * QROWS;

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
        const int64_t rowc = rows[b] < M ? rows[b] : M - 1;
        xrow[b] = x + rowc * ldx + hf * 32;
    }

    // round rd of this wave = group 2 (wave + 4 (rd / 2)) + rd % 2: the two groups of a stage follow each other
    // so that their two scale bytes leave as one 16-bit store.  Software pipeline as in the int4 kernel: the
    // next round's x is in flight while the current one is processed; two register buffers alternate.
    auto group_of = [&](const int rd) { return 2 * (wave + QWAVES * (rd >> 1)) + (rd & 1); };
    const int my_stages = (nstages > wave) ? (nstages - wave + QWAVES - 1) / QWAVES : 0;
    const int rounds = 2 * my_stages;
    uint4 xa[2][4], xb[2][4];
    if (rounds > 0) {
        const int g0 = group_of(0);                      // exists: stage `wave` exists, so group 2 wave < ng
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int s = 0; s < 4; ++s) xa[b][s] = reinterpret_cast<const uint4*>(xrow[b] + g0 * 64)[s];
    }
    __syncthreads();

    uint32_t e_first[2] = {0u, 0u};
    auto round_body = [&](const int rd, uint4 (&xc)[2][4], uint4 (&xn)[2][4], auto PAR) {
        constexpr int parity = decltype(PAR)::value;
        const int g = group_of(rd);
        const bool exists = g < ng;                      // only the second group of the last stage can be missing
        const int gl = exists ? g : ng - 1;
        uint4 bfrag[4][2];
        if (LOWRANK) {
            const uint4* pb = l1p + (size_t)gl * (4 * 2 * 64) + lane;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                bfrag[s][0] = pb[(s * 2 + 0) * 64];
                bfrag[s][1] = pb[(s * 2 + 1) * 64];
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        int gn = (rd + 1 < rounds) ? group_of(rd + 1) : gl;
        if (gn >= ng) gn = ng - 1;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int s = 0; s < 4; ++s) xn[b][s] = reinterpret_cast<const uint4*>(xrow[b] + gn * 64)[s];
        __builtin_amdgcn_sched_barrier(0);

        const float* il_lds = il_s + gl * 64 + hf * 32;
        if (GELU) {
#pragma unroll
            for (int b = 0; b < 2; ++b) gelu_tanh_rows(xc[b]);
        }
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            uint4 codes;
            uint32_t e8;
            quantize_block_mx(xc[b], il_lds, rho, codes, e8);
            if (!exists) e8 = 0u;                        // a group past K: both sides' zero bytes make it contribute 0
            if (exists && rows[b] < M)
                *reinterpret_cast<uint4*>(qx + ((size_t)g * M + rows[b]) * 32 + hf * 16) = codes;
            if (parity == 0) {
                e_first[b] = e8;
            } else if (rows[b] < M) {
                const int st = g >> 1;
                sxe[((size_t)st * M + rows[b]) * 2 + hf] = (uint16_t)(e_first[b] | (e8 << 8));
            }
        }
        if (LOWRANK && exists) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int sidx = 0; sidx < 4; ++sidx) {
                    bf16x8 av = __builtin_bit_cast(bf16x8, xc[b][sidx]);
                    acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8, bfrag[sidx][0]), acc[b], 0, 0, 0);
                    acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8, bfrag[sidx][1]), acc[b], 0, 0, 0);
                }
        }
    };
    for (int rd = 0; rd < rounds; rd += 2) {
        round_body(rd, xa, xb, IC<0>{});
        round_body(rd + 1, xb, xa, IC<1>{});
    }

    if (LOWRANK) {
        __syncthreads();                                     // every wave is done with inv_lambda in LDS
        float* hpart = reinterpret_cast<float*>(smem_raw);   // [4][64][33]
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                int rloc = 32 * b + 8 * (i >> 2) + 4 * hf + (i & 3);
                hpart[(wave * QROWS + rloc) * 33 + rr] = acc[b][i];
            }
        __syncthreads();
        for (int idx = tid; idx < QROWS * r; idx += 256) {
            int rloc = idx / r, j = idx - rloc * r;
            int64_t row = row0 + rloc;
            if (row < M)
                h[row * r + j] = (hpart[(0 * QROWS + rloc) * 33 + j] + hpart[(1 * QROWS + rloc) * 33 + j]) +
                                 (hpart[(2 * QROWS + rloc) * 33 + j] + hpart[(3 * QROWS + rloc) * 33 + j]);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// offline packing of the MXFP4 residual
// ------------------------------------------------------------------------------------------------
__host__ __device__ inline size_t mx_wfrag_bytes(int N, int K) { return (size_t)N * (K / 2); }
__host__ __device__ inline size_t mx_wscale_bytes(int N, int K) { return (size_t)(N / 32) * ((K / 64 + 1) / 2) * 128; }

// Region 1: code fragments [N/32][K/64][64 lanes][16 B], lane (n = lane % 32, kh = lane / 32) holds bytes
// [32 g + 16 kh, +16) of row n of the canonical codes (the A operand of the scaled MFMA as it stands).
// Region 2: scale operands [N/32][stages][64 lanes][2 B]: lane (n, kh) holds the E8M0 bytes of MX blocks
// 2 (2s) + kh and 2 (2s + 1) + kh of channel n, zero for a group past K.
__global__ void pack_weight_mx_kernel(const uint8_t* __restrict__ qw, const uint8_t* __restrict__ sw,
                                      int N, int K, uint8_t* __restrict__ out) {
    const int ng = K >> 6, nst = (ng + 1) >> 1;
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
    uint16_t* o2 = reinterpret_cast<uint16_t*>(out + mx_wfrag_bytes(N, K));
    const size_t n2 = (size_t)(N >> 5) * nst * 64;
    for (size_t v = t0; v < n2; v += stride) {
        const int lane = (int)(v & 63);
        const size_t fr = v >> 6;
        const int st = (int)(fr % nst), nb = (int)(fr / nst);
        const int n = nb * 32 + (lane & 31), kh = lane >> 5;
        uint32_t e = 0;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int g = 2 * st + j;
            if (g < ng) e |= (uint32_t)sw[(size_t)(2 * g + kh) * N + n] << (8 * j);
        }
        o2[v] = (uint16_t)e;
    }
}

// ------------------------------------------------------------------------------------------------
// kernels (b')+(c): block-scaled FP4 GEMM, fused low-rank up-projection, bias, store
// ------------------------------------------------------------------------------------------------
// Block = 4 waves as 2 (tokens) x 2 (channels); a wave owns 64 channels x 32 MT tokens = 2 x MT MFMA tiles.
// The transposed tile D[n][m] is computed (weights are the A operand), as in the int4 kernel.
// Stage = two 64-groups; three-slot LDS ring filled by direct global->LDS loads, protocol as in the int4
// kernel: in the middle of stage s every wave has taken its last operand from the slot, so after the
// barrier the slot takes stage s + 3.
template <int MT, int WNC>
struct MxGeom {
    static constexpr int WAVES = 2 * WNC;                           // 2 (tokens) x WNC (channels)
    static constexpr int BM = 64 * MT;                              // tokens per block
    static constexpr int BN = 64 * WNC;                             // channels per block
    static constexpr uint32_t OFF_A = 0;                            // [group 2][half 2][BM] x 16 B
    static constexpr uint32_t OFF_W = 64 * BM;                      // [group 2][n-block 2 WNC][64 lanes] x 16 B
    static constexpr uint32_t OFF_SX = OFF_W + 4096 * WNC;          // [BM][half 2][group 2] bytes
    static constexpr uint32_t OFF_SW = OFF_SX + 4 * BM;             // [n-block 2 WNC][64 lanes][group 2] bytes
    static constexpr uint32_t STAGE = OFF_SW + 256 * WNC;
    // direct global->LDS loads per wave and stage.  4 waves: MT of A, 2 of W, 1 + 1 of scales;
    // 8 waves: 2 of A, 2 of W, 1 of scales (token scales on waves 0..3, channel scales on waves 4..7)
    static constexpr int NDMA = (WNC == 2) ? MT + 4 : 5;
    static constexpr int NS = (WNC == 2) ? 3 : 4;                   // LDS ring slots: 78 KB (two blocks per CU) or 136 KB (one)
    static_assert(WNC == 2 || (WNC == 4 && MT == 4), "staging is written for 4 waves, or 8 waves with 256 tokens");
};

// The next layer's side of the emitting epilogues.
struct MxNext {
    const float* inv_lambda;     // [N]
    const uint4* l1p;            // packed L1' (K' = N) or null
    uint8_t* qx;                 // [N/64][M][32 B]
    uint8_t* sxe;                // [N/128][M][2][2]
    float* h;                    // [M, r]
    float rho;
    int r;
};

// Kernel (a') of the NEXT layer on a wave's finished tile (64 channels nw .. nw + 63 of tokens mw .. mw + 32 MT - 1):
// round to bf16 (what the layer would have stored), optionally GELU, trade n-blocks between lanes l and l + 32 so
// that a lane holds one whole MX block of its token, quantise it with the quantise kernel's own function, write
// codes and scale byte.  If the next layer has a low-rank branch, hp[mi] returns the wave's share of h' for its
// tokens ([token][j] in the accumulator layout: lane holds column j = lane % 32).
template <int MT, bool GELU>
__device__ __forceinline__ void emit_next_mx(const float16v (&y)[2][MT], const MxNext& nx, int64_t M, int64_t mw, int nw,
                                             int lane, float16v (&hp)[MT]) {
    const int l32 = lane & 31, kh = lane >> 5;
    const int gq = nw >> 6;                                    // this wave's 64-group of the next layer
    const float* il = nx.inv_lambda + nw + kh * 32;
    uint4 bfrag[4][2];
    if (nx.r > 0) {
        const uint4* pb = nx.l1p + (size_t)gq * (4 * 2 * 64) + lane;
#pragma unroll
        for (int sI = 0; sI < 4; ++sI) {
            bfrag[sI][0] = pb[(sI * 2 + 0) * 64];
            bfrag[sI][1] = pb[(sI * 2 + 1) * 64];
        }
    }
#pragma unroll
    for (int mi = 0; mi < MT; ++mi) {
        // register 4 q + j of y[ni][mi] is channel 32 ni + 8 q + 4 kh + j of token mw + 32 mi + l32
        uint32_t pk[2][8];
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int d = 0; d < 8; ++d) {
                uint32_t w = f2_bf16_rne(y[ni][mi][2 * d], y[ni][mi][2 * d + 1]);
                if (GELU) w = gelu_tanh_bf16x2(w);
                pk[ni][d] = w;
            }
        uint4 xc[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            // first result: own value in lanes 0..31, the lower lanes' second operand in lanes 32..63;
            // second result: the upper lanes' first operand in lanes 0..31, own value in lanes 32..63
            const auto e0 = __builtin_amdgcn_permlane32_swap(pk[0][2 * q], pk[1][2 * q], false, false);
            const auto e1 = __builtin_amdgcn_permlane32_swap(pk[0][2 * q + 1], pk[1][2 * q + 1], false, false);
            xc[q] = uint4{e0[0], e1[0], e0[1], e1[1]};         // channels 32 kh + 8 q + 0..7: MX block 2 gq + kh
        }
        uint4 codes;
        uint32_t e8;
        quantize_block_mx(xc, il, nx.rho, codes, e8);
        const int64_t row = mw + mi * 32 + l32;
        if (row < M) {
            *reinterpret_cast<uint4*>(nx.qx + ((size_t)gq * M + row) * 32 + kh * 16) = codes;
            nx.sxe[(((size_t)(gq >> 1) * M + row) * 2 + kh) * 2 + (gq & 1)] = (uint8_t)e8;
        }
        if (nx.r > 0) {
            float16v acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
#pragma unroll
            for (int sI = 0; sI < 4; ++sI) {
                const bf16x8 av = __builtin_bit_cast(bf16x8, xc[sI]);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8, bfrag[sI][0]), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8, bfrag[sI][1]), acc, 0, 0, 0);
            }
            hp[mi] = acc;
        }
    }
}

// The WNC waves of a block that share tokens (wn = 0 .. WNC - 1, same wm) sum their shares of h' through LDS, one
// after the other into the same area (`part`: this wm's [MT * 16][64] floats, block-uniform control flow), and wave
// wn = 0 adds the block's sum to the zeroed h' with atomic adds.  Register (mi, i) of lane (l32, kh) is token
// mw + 4 kh + [32 mi + 8 (i / 4) + i % 4], column l32.
template <int MT, int WNC>
__device__ __forceinline__ void add_next_h(float16v (&hp)[MT], float* part, int wn, const MxNext& nx, int64_t M, int64_t mw,
                                           int lane) {
    const int l32 = lane & 31, kh = lane >> 5;
    part += lane;
#pragma unroll
    for (int w = WNC - 1; w >= 1; --w) {
        if (wn == w) {
#pragma unroll
            for (int mi = 0; mi < MT; ++mi)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float v = hp[mi][i];
                    if (w != WNC - 1) v += part[(mi * 16 + i) * 64];
                    part[(mi * 16 + i) * 64] = v;
                }
        }
        __syncthreads();
    }
    if (wn == 0) {
#pragma unroll
        for (int mi = 0; mi < MT; ++mi)
#pragma unroll
            for (int i = 0; i < 16; ++i) hp[mi][i] += part[(mi * 16 + i) * 64];
        const int64_t first = mw + 4 * kh;
        const int left = (l32 < nx.r && first < M) ? (int)((M - first < 32 * MT) ? M - first : 32 * MT) : 0;
        float* hb = nx.h + first * nx.r + l32;
#pragma unroll
        for (int mi = 0; mi < MT; ++mi)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int rl = 32 * mi + 8 * (i >> 2) + (i & 3);
                if (rl < left) unsafeAtomicAdd(hb + rl * nx.r, hp[mi][i]);
            }
    }
}

// MODE: MX_LAYER stores y.  MX_NEXT / MX_NEXT_GELU (four-wave geometry only): y never reaches HBM; the wave rounds
// its tile to bf16, optionally applies GELU and runs the NEXT layer's kernel (a') on it.  A wave's 64 channels are two
// MX blocks of the next layer's K axis: after lanes l and l + 32 have traded n-blocks a lane holds one whole block
// of its token, so the shared exponent and the codes need no further exchange; the wave's share of
// h' = x^' L1' is added to the zeroed h' with atomic adds (after the two waves that share tokens have been summed
// in LDS).
enum { MX_LAYER = 0, MX_NEXT = 1, MX_NEXT_GELU = 2 };

template <int MT, int WNC, int MODE>
__global__ __launch_bounds__(128 * WNC, (WNC == 2) ? 2 : 1)
void gemm_mx_kernel(const uint8_t* __restrict__ qx, const uint16_t* __restrict__ sxe,
                    const uint4* __restrict__ wfrag, const uint16_t* __restrict__ wscale,
                    const float* __restrict__ h, const uint16_t* __restrict__ L2, const float* __restrict__ bias,
                    int64_t M, int N, int K, int r, void* __restrict__ yout, int64_t ldy, int out_f32,
                    const TileGrid tg, const MxNext nx) {
    static_assert(MODE == MX_LAYER || WNC == 2, "the emitting epilogue is written for the four-wave geometry");
    using G = MxGeom<MT, WNC>;
    constexpr int BM = G::BM;
    constexpr int NDMA = G::NDMA;
    constexpr int NS = G::NS;
    __shared__ __attribute__((aligned(16))) uint8_t ring[NS * G::STAGE];

    int mt, nt;                                 // XCD-aware tile order (svdq_tiles.h)
    if (!tile_of(tg, blockIdx.x, mt, nt)) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int l32 = lane & 31, kh = lane >> 5;
    const int ng = K >> 6;
    const int nstages = (ng + 1) >> 1;
    const int64_t m0 = (int64_t)mt * BM;
    const int n0 = nt * G::BN;
    const int nbB = n0 >> 5;
    const uint32_t ring0 = (uint32_t)(uintptr_t)(lds_byte*)ring;

    // ---- staging.  4 waves: wave w moves, per stage, the A chunks (group w / 2, half w % 2, 64-token quarter
    // q = 0..MT-1), the W chunks (group w / 2, n-blocks 2 (w % 2) + {0, 1}), 64 tokens' scale bytes and one half of
    // the channel scale bytes (waves 2, 3 repeat what waves 0, 1 move so that every wave counts NDMA loads).
    // 8 waves: A chunks (group w / 4, half (w / 2) % 2, quarters 2 (w % 2) + {0, 1}), W chunks (group w / 4,
    // n-blocks 2 (w % 4) + {0, 1}), and one scale transfer: tokens [64 w, +64) on waves 0..3, n-block pair w - 4 on 4..7.
    constexpr int NA = (WNC == 2) ? MT : 2;
    const int cj = (WNC == 2) ? (wave >> 1) : (wave >> 2);
    const int sp = (WNC == 2) ? (wave & 1) : ((wave >> 1) & 1);
    const int q0 = (WNC == 2) ? 0 : 2 * (wave & 1);
    const int nb0 = (WNC == 2) ? 2 * (wave & 1) : 2 * (wave & 3);
    uint32_t va[NA];
#pragma unroll
    for (int q = 0; q < NA; ++q) {
        const int64_t row = m0 + (q0 + q) * 64 + lane;
        va[q] = (uint32_t)(((row < M) ? row : (M - 1)) * 32 + sp * 16);
    }
    const uint32_t vl16 = lane * 16;
    const uint32_t vw[2] = {(uint32_t)((nb0 + 0) * ng * 1024) + vl16, (uint32_t)((nb0 + 1) * ng * 1024) + vl16};
    const int sxw = (WNC == 2) ? ((wave < MT) ? wave : wave - MT) : (wave & 3);   // 64-token quarter whose scales this wave moves
    uint32_t vsx;
    {
        const int64_t row = m0 + sxw * 64 + lane;
        vsx = (uint32_t)(((row < M) ? row : (M - 1)) * 4);
    }
    const int swp = (WNC == 2) ? (wave & 1) : (wave & 3);             // pair of n-blocks whose scales this wave moves
    const uint32_t vsw = (uint32_t)(kh * nstages * 128 + l32 * 4);    // channel scales: lanes 0..31 one n-block, 32..63 the next
    // eight waves: this wave's one scale transfer per stage (token scales on waves 0..3, channel scales on 4..7)
    const uint32_t vsc = (wave < 4) ? vsx : vsw;
    const uint8_t* sc_base = (wave < 4) ? reinterpret_cast<const uint8_t*>(sxe)
                                        : reinterpret_cast<const uint8_t*>(wscale + (size_t)(nbB + 2 * swp) * nstages * 64);
    const size_t sc_stride = (wave < 4) ? (size_t)M * 4 : (size_t)128;
    const uint32_t sc_lds = (wave < 4) ? G::OFF_SX + sxw * 256 : G::OFF_SW + swp * 256;
    // transfer p (0 .. NDMA - 1) of this wave for stage s; always requested in this order.  Eight waves: the one scale
    // transfer's base, stride and destination were chosen before the loop, so it needs no wave-dependent branch.
    auto stage_piece = [&](const int s, const uint32_t slot, const int p) {
        const int g = (2 * s + cj < ng) ? 2 * s + cj : ng - 1;        // odd tail: re-read (its scale bytes are zero)
        if (p < NA) dma16(qx + (size_t)g * M * 32, va[p], slot + G::OFF_A + ((cj * 2 + sp) * BM + (q0 + p) * 64) * 16);
        else if (p < NA + 2) dma16(wfrag + ((size_t)nbB * ng + g) * 64, vw[p - NA], slot + G::OFF_W + (cj * 2 * WNC + nb0 + p - NA) * 1024);
        else if (WNC == 4) dma4(sc_base + (size_t)s * sc_stride, vsc, slot + sc_lds);
        else if (p == NA + 2) dma4(sxe + (size_t)s * M * 2, vsx, slot + G::OFF_SX + sxw * 256);
        else dma4(wscale + ((size_t)(nbB + 2 * swp) * nstages + s) * 64, vsw, slot + G::OFF_SW + swp * 256);
    };
    auto stage_issue = [&](const int s) {
        const uint32_t slot = ring0 + (uint32_t)(s % NS) * G::STAGE;
#pragma unroll
        for (int p = 0; p < NDMA; ++p) stage_piece(s, slot, p);
    };

    // per-lane LDS read offsets inside a slot
    const uint32_t rd_a = G::OFF_A + (kh * BM + wm * (32 * MT) + l32) * 16;   // + group 32 BM + mi 512
    const uint32_t rd_w = G::OFF_W + (wn * 2 * 64 + lane) * 16;               // + group 2048 WNC + ni 1024
    const uint32_t rd_sx = G::OFF_SX + ((wm * (32 * MT) + l32) * 2 + kh) * 2; // + mi 128
    const uint32_t rd_sw = G::OFF_SW + (wn * 2 * 64 + lane) * 2;              // + ni 128

    float16v y[2][MT];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) y[a][b][i] = 0.0f;

    // wait until at most k stages' worth of this wave's transfers are outstanding (k = 0 .. NS - 1)
    auto wait_stages = [&](const int k) {
        if (k <= 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        else if (k == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NDMA) : "memory");
        else if (k == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * NDMA) : "memory");
        else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(3 * NDMA) : "memory");
    };
    const int64_t mw = m0 + wm * (32 * MT);                   // first token of this wave's tile
    {
        // the first stages are requested; while they are in flight y starts as the low-rank term plus the bias
        // (eq. 7, 11), so that the latency of those loads hides here instead of standing at the end of the tile
        const int pre = nstages < NS ? nstages : NS;
        for (int s = 0; s < pre; ++s) stage_issue(s);
        add_lowrank_bias<2, MT>(y, h, L2, bias, mw, n0 + wn * 64, M, N, r, lane);
        wait_stages(pre - 1);
    }
    __syncthreads();

    // Two operand register sets: set 0 feeds the first group of a stage (scale byte 0 of each 16-bit scale
    // entry), set 1 the second (byte 1).  Each set is requested from LDS one group ahead of its MFMAs, so the
    // loads of one group land while the other group's eight matrix instructions run.
    struct Operands {
        uint4 wf[2], xf[MT];
        uint32_t sw[2], sx[MT];
    };
    Operands op0, op1;
    auto fetch = [&](Operands& o, const uint32_t slot, const int j) {
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            o.wf[ni] = lds_read16_pinned(slot + rd_w + j * 2048 * WNC + ni * 1024);
            o.sw[ni] = lds_read2_pinned(slot + rd_sw + ni * 128);
        }
#pragma unroll
        for (int mi = 0; mi < MT; ++mi) {
            o.xf[mi] = lds_read16_pinned(slot + rd_a + j * 32 * BM + mi * 512);
            o.sx[mi] = lds_read2_pinned(slot + rd_sx + mi * 128);
        }
    };
    auto mma_group = [&](const Operands& o, auto JC) {
        constexpr int j = decltype(JC)::value;
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const int8v a = {(int)o.wf[ni].x, (int)o.wf[ni].y, (int)o.wf[ni].z, (int)o.wf[ni].w, 0, 0, 0, 0};
#pragma unroll
            for (int mi = 0; mi < MT; ++mi) {
                const int8v b = {(int)o.xf[mi].x, (int)o.xf[mi].y, (int)o.xf[mi].z, (int)o.xf[mi].w, 0, 0, 0, 0};
                y[ni][mi] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, y[ni][mi], 4, 4, j, (int)o.sw[ni], j, (int)o.sx[mi]);
            }
        }
    };

    // The eight matrix instructions of a group carry, between them, the LDS reads of the OTHER operand set (two per
    // instruction) and, in a stage's second group, the slot's new transfer requests (one each).  Requested as a burst
    // ahead of a group they are time in which the matrix pipe has nothing queued: the waves of a block run in step.
    auto mma_with_fetch = [&](const Operands& o, auto JC, Operands& on, const uint32_t slot, const int jn, auto request) {
        constexpr int j = decltype(JC)::value;
        auto one = [&](auto TC) {
            constexpr int t = decltype(TC)::value, ni = t / MT, mi = t % MT;
            const int8v a = {(int)o.wf[ni].x, (int)o.wf[ni].y, (int)o.wf[ni].z, (int)o.wf[ni].w, 0, 0, 0, 0};
            const int8v b = {(int)o.xf[mi].x, (int)o.xf[mi].y, (int)o.xf[mi].z, (int)o.xf[mi].w, 0, 0, 0, 0};
            y[ni][mi] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, y[ni][mi], 4, 4, j, (int)o.sw[ni], j, (int)o.sx[mi]);
            __builtin_amdgcn_sched_barrier(0);
            if (t < NDMA) request(t);
            if (t < 2) {
                on.wf[t] = lds_read16_pinned(slot + rd_w + jn * 2048 * WNC + t * 1024);
                on.sw[t] = lds_read2_pinned(slot + rd_sw + t * 128);
            } else if (t < 2 + MT) {
                on.xf[t - 2] = lds_read16_pinned(slot + rd_a + jn * 32 * BM + (t - 2) * 512);
                on.sx[t - 2] = lds_read2_pinned(slot + rd_sx + (t - 2) * 128);
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        static_assert(MT == 4 && NDMA <= 8, "eight instructions per group");
        one(IC<0>{}); one(IC<1>{}); one(IC<2>{}); one(IC<3>{});
        one(IC<4>{}); one(IC<5>{}); one(IC<6>{}); one(IC<7>{});
    };

    // One stage.  FULL: stages s+1..s+NS exist, so the body is straight-line code (the compiler otherwise sinks
    // the first group's matrix instructions past the conditional blocks, next to the second group's).
    auto stage_body = [&](const int s, const uint32_t cur, const uint32_t nxt, auto FULLC) {
        constexpr bool FULL = decltype(FULLC)::value;
        if (FULL) {
            // first group multiplied while the second group's operands are requested: after it this wave has
            // requested everything it needs from the slot (the barrier waits for the loads to return), so after the
            // barrier the slot can take stage s + NS; stage s + 1, requested NS - 1 stages ago, is made visible for
            // the reads of the second group's instructions (stages s + 2 .. s + NS - 1 may stay in flight)
            mma_with_fetch(op0, IC<0>{}, op1, cur, 1, [](int) {});
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * NDMA) : "memory");
            __syncthreads();
            mma_with_fetch(op1, IC<1>{}, op0, nxt, 0, [&](const int p) { stage_piece(s + NS, cur, p); });
            return;
        }
        // the last stages, with their conditions
        fetch(op1, cur, 1);
        __builtin_amdgcn_sched_barrier(0);
        mma_group(op0, IC<0>{});
        __builtin_amdgcn_sched_barrier(0);
        if (s + 1 < nstages) {
            wait_stages((nstages - 1 < s + NS - 1 ? nstages - 1 : s + NS - 1) - (s + 1));
            __syncthreads();
            if (s + NS < nstages) stage_issue(s + NS);
            fetch(op0, nxt, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        mma_group(op1, IC<1>{});
        __builtin_amdgcn_sched_barrier(0);
    };
    fetch(op0, ring0, 0);
    uint32_t cur = ring0;
    auto next_slot = [&](const uint32_t c) { return (c == ring0 + (NS - 1) * G::STAGE) ? ring0 : c + G::STAGE; };
    int s = 0;
    for (; s + NS < nstages; ++s) {
        const uint32_t nxt = next_slot(cur);
        stage_body(s, cur, nxt, IC<1>{});
        cur = nxt;
    }
    for (; s < nstages; ++s) {
        const uint32_t nxt = next_slot(cur);
        stage_body(s, cur, nxt, IC<0>{});
        cur = nxt;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // nothing may still be writing this block's LDS when it ends

    // ---- epilogue (c): store (the low-rank term and the bias are already in y)
    if constexpr (MODE != MX_LAYER) {
        float16v hp[MT];
        emit_next_mx<MT, MODE == MX_NEXT_GELU>(y, nx, M, mw, n0 + wn * 64, lane, hp);
        if (nx.r > 0) {
            __syncthreads();                                   // every wave is done with the operand ring
            add_next_h<MT, WNC>(hp, reinterpret_cast<float*>(ring) + wm * (MT * 16 * 64), wn, nx, M, mw, lane);
        }
        return;
    }
    if (out_f32) {
        store_tile_f32<2, MT>(y, reinterpret_cast<float*>(yout), ldy, mw, n0 + wn * 64, M, lane);
    } else {
        __syncthreads();                                       // every wave is done with the operand ring
        uint16_t* yw = reinterpret_cast<uint16_t*>(yout) + mw * ldy + n0 + wn * 64;
        if (WNC == 2) {
            store_tile_bf16<MT>([&](int ni, int mi, int i) { return y[ni][mi][i]; },
                                ring0 + wave * (32 * MT) * YROW, lane, yw, ldy, M - mw);
        } else {                                               // eight waves: 64 tokens at a time fit the ring
            constexpr int HM = MT / 2;
            store_tile_bf16<HM>([&](int ni, int mi, int i) { return y[ni][mi][i]; },
                                ring0 + wave * (32 * HM) * YROW, lane, yw, ldy, M - mw);
            store_tile_bf16<HM>([&](int ni, int mi, int i) { return y[ni][mi + HM][i]; },
                                ring0 + wave * (32 * HM) * YROW, lane, yw + (int64_t)(32 * HM) * ldy, ldy, M - mw - 32 * HM);
        }
    }
}


// The eight-wave kernel as ONE block per CU that walks its tiles.  A block that is alone on its CU shows every
// tile's start and end: filling the ring (12 k clocks when all CUs of a round of blocks ask at once) and the
// store (6 k) stand beside a K loop of 62 k.  Here the ring never drains between tiles: the slots that the last
// stages of a tile hand over take the first stages of the block's NEXT tile, so those arrive during the end of the
// loop and the store, and the store transposes through its own LDS area behind a three-slot ring.  Tiles are taken
// in the same XCD-aware order (tile ids b, b + gridDim, ...; gridDim a multiple of 8 keeps a block on one XCD's
// share).  Same arithmetic, same order of operations per output as gemm_mx_kernel.
//
// The low-rank term's h rows (eq. 7: 256 tokens x r binary32 per tile) were what a tile start waited for longest:
// sixteen 16-byte loads per lane, requested behind the previous tile's stores (measured: 6-7 % of the kernel at
// K = 5120).  They now travel like the operands: the first two stages of a tile request the NEXT tile's rows into an
// LDS area of their own, in the instruction slots of the second group that carry no operand request, and the tile
// start reads them from there.  A token has eight 16-byte places there (128 bytes, r = 32; with r = 16 the upper four
// hold nothing of use); piece c of token t sits at place c ^ ((t >> 1) & (r / 4 - 1)): a lane reads one piece of its
// own token, and with the pieces rotated by token the 32 tokens of an instruction spread over the banks.  To make
// room the store transposes one 32 x 32 accumulator block at a time (rows of 64 bytes, padded to 80).
template <int MT>
__global__ __launch_bounds__(512, 1)
void gemm_mx_persistent_kernel(const uint8_t* __restrict__ qx, const uint16_t* __restrict__ sxe,
                               const uint4* __restrict__ wfrag, const uint16_t* __restrict__ wscale,
                               const float* __restrict__ h, const uint16_t* __restrict__ L2, const float* __restrict__ bias,
                               int64_t M, int N, int K, int r, void* __restrict__ yout, int64_t ldy, int out_f32,
                               const TileGrid tg) {
    constexpr int WNC = 4;
    using G = MxGeom<MT, WNC>;
    constexpr int BM = G::BM, NDMA = G::NDMA, NS = 3;
    constexpr uint32_t YROW32 = 80;                                   // 32 channels of a token as bf16 + 16 bytes of padding
    constexpr uint32_t STORE_BYTES = 32 * YROW32;                     // per wave: one 32-token x 32-channel block at a time
    constexpr uint32_t HBUF = (uint32_t)BM * 128;                     // the tile's h rows, r <= 32
    __shared__ __attribute__((aligned(16))) uint8_t ring[NS * G::STAGE + 2 * WNC * STORE_BYTES + HBUF];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int l32 = lane & 31, kh = lane >> 5;
    const int ng = K >> 6;
    const int nstages = (ng + 1) >> 1;                                // >= NS + 2 (the launcher sees to it)
    const uint32_t ring0 = (uint32_t)(uintptr_t)(lds_byte*)ring;
    const uint32_t store0 = ring0 + NS * G::STAGE + wave * STORE_BYTES;
    const uint32_t hbuf0 = ring0 + NS * G::STAGE + 2 * WNC * STORE_BYTES;
    const int ptm = (r >> 2) - 1;                                     // 16-byte pieces per token of h, less one; r is 0, 16 or 32
    constexpr int H_TRANSFERS = 4;                                    // 1-KB transfers per wave and tile: BM x 128 bytes over 8 waves

    // tile ids: the one-tile kernel's order (svdq_tiles.h), of which this block takes ids b, b + gridDim, ...
    const int total = tile_ids(tg);
    auto decode = [&](const int id, int& mt, int& nt) { return tile_of(tg, id, mt, nt); };
    auto next_valid = [&](int id) {
        for (id += gridDim.x; id < total; id += gridDim.x) {
            int mt, nt;
            if (decode(id, mt, nt)) return id;
        }
        return -1;
    };

    // ---- staging (the eight-wave assignment of gemm_mx_kernel); what depends on the tile sits in TileAddr
    const int cj = wave >> 2, sp = (wave >> 1) & 1, q0 = 2 * (wave & 1), nb0 = 2 * (wave & 3);
    const int sxw = wave & 3, swp = wave & 3;
    const uint32_t vl16 = lane * 16;
    const uint32_t vw[2] = {(uint32_t)((nb0 + 0) * ng * 1024) + vl16, (uint32_t)((nb0 + 1) * ng * 1024) + vl16};
    const uint32_t vsw = (uint32_t)(kh * nstages * 128 + l32 * 4);
    const size_t sc_stride = (wave < 4) ? (size_t)M * 4 : (size_t)128;
    const uint32_t sc_lds = (wave < 4) ? G::OFF_SX + sxw * 256 : G::OFF_SW + swp * 256;
    struct TileAddr {
        uint32_t va[2], vsc;
        const uint8_t* sc_base;
        int64_t m0;
        int n0, nbB;
    };
    auto tile_addr = [&](const int id) {
        int mt, nt;
        decode(id, mt, nt);
        TileAddr t;
        t.m0 = (int64_t)mt * BM;
        t.n0 = nt * G::BN;
        t.nbB = t.n0 >> 5;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int64_t row = t.m0 + (q0 + q) * 64 + lane;
            t.va[q] = (uint32_t)(((row < M) ? row : (M - 1)) * 32 + sp * 16);
        }
        const int64_t srow = t.m0 + sxw * 64 + lane;
        t.vsc = (wave < 4) ? (uint32_t)(((srow < M) ? srow : (M - 1)) * 4) : vsw;
        t.sc_base = (wave < 4) ? reinterpret_cast<const uint8_t*>(sxe)
                               : reinterpret_cast<const uint8_t*>(wscale + (size_t)(t.nbB + 2 * swp) * nstages * 64);
        return t;
    };
    // transfer p (0 .. NDMA - 1) of this wave for stage s of tile t; always requested in this order
    auto stage_piece = [&](const TileAddr& t, const int s, const uint32_t slot, const int p) {
        const int g = (2 * s + cj < ng) ? 2 * s + cj : ng - 1;        // odd tail: re-read (its scale bytes are zero)
        if (p < 2) dma16(qx + (size_t)g * M * 32, t.va[p], slot + G::OFF_A + ((cj * 2 + sp) * BM + (q0 + p) * 64) * 16);
        else if (p < 4) dma16(wfrag + ((size_t)t.nbB * ng + g) * 64, vw[p - 2], slot + G::OFF_W + (cj * 2 * WNC + nb0 + p - 2) * 1024);
        else dma4(t.sc_base + (size_t)s * sc_stride, t.vsc, slot + sc_lds);
    };
    auto stage_issue = [&](const TileAddr& t, const int s, const uint32_t slot) {
#pragma unroll
        for (int p = 0; p < NDMA; ++p) stage_piece(t, s, slot, p);
    };
    // transfer i (0 .. H_TRANSFERS - 1) of this wave for the h rows of the tile whose first token is m0: eight tokens,
    // lane l fills place l % 8 of token l / 8 (a place that holds nothing of use re-reads a piece that exists).  No
    // branch: a stage must stay one basic block, or the compiler moves its matrix instructions out of their places.
    // With r = 0 the launcher passes some readable address as h, and the lanes read within its first 128 bytes.
    auto h_request = [&](const int64_t m0, const int i) {
        int ln = lane;
        asm volatile("" : "+v"(ln));                                  // the address arithmetic stays where the request is
        const int j = wave * H_TRANSFERS + i;
        const int t = j * 8 + (ln >> 3);
        const int c = ((ln & 7) ^ (t >> 1)) & ptm & 7;
        const int64_t left = M - 1 - m0;                              // rows beyond M: the last row again
        const int row = (t < left) ? t : (int)left;
        dma16(h + m0 * r, (uint32_t)(row * r * 4 + c * 16), hbuf0 + j * 1024);
    };

    const uint32_t rd_a = G::OFF_A + (kh * BM + wm * (32 * MT) + l32) * 16;
    const uint32_t rd_w = G::OFF_W + (wn * 2 * 64 + lane) * 16;
    const uint32_t rd_sx = G::OFF_SX + ((wm * (32 * MT) + l32) * 2 + kh) * 2;
    const uint32_t rd_sw = G::OFF_SW + (wn * 2 * 64 + lane) * 2;

    struct Operands {
        uint4 wf[2], xf[MT];
        uint32_t sw[2], sx[MT];
    };
    Operands op0, op1;
    auto fetch = [&](Operands& o, const uint32_t slot, const int j) {
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            o.wf[ni] = lds_read16_pinned(slot + rd_w + j * 2048 * WNC + ni * 1024);
            o.sw[ni] = lds_read2_pinned(slot + rd_sw + ni * 128);
        }
#pragma unroll
        for (int mi = 0; mi < MT; ++mi) {
            o.xf[mi] = lds_read16_pinned(slot + rd_a + j * 32 * BM + mi * 512);
            o.sx[mi] = lds_read2_pinned(slot + rd_sx + mi * 128);
        }
    };
    float16v y[2][MT];
    auto mma_group = [&](const Operands& o, auto JC) {
        constexpr int j = decltype(JC)::value;
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const int8v a = {(int)o.wf[ni].x, (int)o.wf[ni].y, (int)o.wf[ni].z, (int)o.wf[ni].w, 0, 0, 0, 0};
#pragma unroll
            for (int mi = 0; mi < MT; ++mi) {
                const int8v b = {(int)o.xf[mi].x, (int)o.xf[mi].y, (int)o.xf[mi].z, (int)o.xf[mi].w, 0, 0, 0, 0};
                y[ni][mi] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, y[ni][mi], 4, 4, j, (int)o.sw[ni], j, (int)o.sx[mi]);
            }
        }
    };
    auto next_slot = [&](const uint32_t c) { return (c == ring0 + (NS - 1) * G::STAGE) ? ring0 : c + G::STAGE; };

    int id = blockIdx.x;
    {
        int mt, nt;
        if (!decode(id, mt, nt)) id = next_valid(id);
    }
    if (id < 0) return;
    TileAddr T = tile_addr(id);
    uint32_t cur = ring0;                                             // slot of the current tile's stage 0
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) h_request(T.m0, i);         // the first tile's h rows: requested first, awaited below
        uint32_t sl = cur;
        for (int s = 0; s < NS; ++s) {
            stage_issue(T, s, sl);
            sl = next_slot(sl);
        }
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NS * NDMA) : "memory");
        __syncthreads();
    }

    // What a stage does once its first group is multiplied: the stage after it (of this tile or of the next) is awaited
    // and made visible, and the slot takes stage s + NS of this tile (SAME) or, when the tile has no such stage left,
    // stage s + NS - nstages of the block's next tile (NEXT).  END: the tile's last stage, whose successor's operands
    // the next tile requests itself.  The block's last tile "prefetches" its own first stages again: three stages
    // nobody reads, for a loop without a third variant.
    while (true) {
        const int nid = next_valid(id);
        const TileAddr T1 = tile_addr(nid >= 0 ? nid : id);
        const int64_t mw = T.m0 + wm * (32 * MT);
        // the per-lane address arithmetic of the low-rank term and of the store is the same for every tile; hidden
        // from the compiler here, it is redone per tile instead of being kept in (spilled) registers across the K loops
        int lane_t = lane;
        asm volatile("" : "+v"(lane_t));
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < MT; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) y[a][b][i] = 0.0f;
        // y starts as the low-rank term plus the bias (eq. 7, 11).  The tile's h rows are in LDS: requested during the
        // previous tile's first stages (by every wave, each of which has since waited for younger transfers and passed
        // barriers), or before the loop for the block's first tile.
        const int th = wm * (32 * MT) + (lane_t & 31);               // this lane's token of block 0; the rotation is the same for
        const int rot = (th >> 1) & ptm;                             // all its blocks (32 tokens apart)
        const uint32_t hrow = hbuf0 + th * 128;
        add_lowrank_bias_from<2, MT>(y, [&](const int mi, const int k) {
            const uint4 v = lds_read16(hrow + (((k >> 2) ^ rot) << 4) + mi * (32 * 128));
            return float4{__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
        }, L2, bias, T.n0 + wn * 64, N, r, lane_t);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 1) * NDMA) : "memory");    // stage 0 of this tile
        __syncthreads();
        fetch(op0, cur, 0);

        // The eight matrix instructions of a group carry the LDS reads of the OTHER operand set between them, two per
        // instruction: both waves of a SIMD belong to this block and run in step, so a burst of twelve reads (or the
        // five transfer requests) ahead of a group is time in which the matrix pipe has nothing queued.
        auto mma_with_fetch = [&](const Operands& o, auto JC, Operands& on, const uint32_t slot, const int jn, const bool doit,
                                  auto request) {
            constexpr int j = decltype(JC)::value;
            auto one = [&](auto TC) {
                constexpr int t = decltype(TC)::value, ni = t / MT, mi = t % MT;
                const int8v a = {(int)o.wf[ni].x, (int)o.wf[ni].y, (int)o.wf[ni].z, (int)o.wf[ni].w, 0, 0, 0, 0};
                const int8v b = {(int)o.xf[mi].x, (int)o.xf[mi].y, (int)o.xf[mi].z, (int)o.xf[mi].w, 0, 0, 0, 0};
                y[ni][mi] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, y[ni][mi], 4, 4, j, (int)o.sw[ni], j, (int)o.sx[mi]);
                __builtin_amdgcn_sched_barrier(0);
                request(t);
                if (doit) {
                    if (t < 2) {
                        on.wf[t] = lds_read16_pinned(slot + rd_w + jn * 2048 * WNC + t * 1024);
                        on.sw[t] = lds_read2_pinned(slot + rd_sw + t * 128);
                    } else if (t < 2 + MT) {
                        on.xf[t - 2] = lds_read16_pinned(slot + rd_a + jn * 32 * BM + (t - 2) * 512);
                        on.sx[t - 2] = lds_read2_pinned(slot + rd_sx + (t - 2) * 128);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            };
            static_assert(MT == 4 && NDMA <= 8, "eight instructions per group");
            one(IC<0>{}); one(IC<1>{}); one(IC<2>{}); one(IC<3>{});
            one(IC<4>{}); one(IC<5>{}); one(IC<6>{}); one(IC<7>{});
        };
        // Between the two groups of a stage stand only the wait and the barrier: the stage after this one is awaited
        // and made visible, and this stage's slot is free (every read of it was requested during the first group).
        // The second group's instructions then also carry the slot's new transfer requests, one each.
        // HC >= 0: the instructions left over also request transfers HC, HC + 1, ... of the NEXT tile's h rows.  These
        // are younger than the operand transfers the waits count, so every wait holds for at least what it names.
        auto stage_body = [&](const int s, const uint32_t c, const uint32_t nxt, auto SAMEC, auto ENDC, auto HCC) {
            constexpr bool SAME = decltype(SAMEC)::value, END = decltype(ENDC)::value;
            constexpr int HC = decltype(HCC)::value;
            mma_with_fetch(op0, IC<0>{}, op1, c, 1, true, [](int) {});
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * NDMA) : "memory");
            __syncthreads();
            mma_with_fetch(op1, IC<1>{}, op0, nxt, 0, !END, [&](const int p) {
                if (p >= NDMA) {
                    if (HC >= 0) h_request(T1.m0, HC + p - NDMA);
                } else if (SAME) stage_piece(T, s + NS, c, p);
                else stage_piece(T1, s + NS - nstages, c, p);
            });
        };
        int s = 0;
        {
            static_assert(NDMA == 5, "three free instructions per stage: the four h transfers take two stages");
            uint32_t nxt = next_slot(cur);
            stage_body(0, cur, nxt, IC<1>{}, IC<0>{}, IC<0>{});
            cur = nxt;
            nxt = next_slot(cur);
            stage_body(1, cur, nxt, IC<1>{}, IC<0>{}, IC<3>{});
            cur = nxt;
            s = 2;
        }
        for (; s + NS < nstages; ++s) {
            const uint32_t nxt = next_slot(cur);
            stage_body(s, cur, nxt, IC<1>{}, IC<0>{}, IC<-1>{});
            cur = nxt;
        }
        for (; s + 1 < nstages; ++s) {
            const uint32_t nxt = next_slot(cur);
            stage_body(s, cur, nxt, IC<0>{}, IC<0>{}, IC<-1>{});
            cur = nxt;
        }
        stage_body(s, cur, next_slot(cur), IC<0>{}, IC<1>{}, IC<-1>{});
        cur = next_slot(cur);                                         // where the next tile's stage 0 went

        // ---- store: the ring belongs to the next tile by now, so the transposition uses the area behind it.  (The
        // emitting epilogues stay with the four-wave kernel: alone on its CU a block would run their vector-ALU work,
        // about 10 k clocks per tile, beside nothing; measured 1.83 ms against 1.58 ms for the C3 up-projection.)
        int lane_s = lane;
        asm volatile("" : "+v"(lane_s));                              // the store's address arithmetic stays behind the K loop
        if (out_f32) {
            store_tile_f32<2, MT>(y, reinterpret_cast<float*>(yout), ldy, mw, T.n0 + wn * 64, M, lane_s);
        } else {
            uint16_t* yw = reinterpret_cast<uint16_t*>(yout) + mw * ldy + T.n0 + wn * 64;
            // One accumulator block (32 tokens x 32 channels) at a time through this wave's LDS region: a lane writes its
            // token's 4-channel pieces, then four lanes store a token's 64 bytes.  Software-pipelined: a block's two
            // reads are requested together, and the NEXT block is converted and written behind them, before the wait
            // for their data -- LDS serves a wave's requests in order, so the reads see the old block and the writes
            // land after them.  (One read, wait, store at a time, the 32 LDS round trips were the whole store phase.)
            const int l32s = lane_s & 31, khs = lane_s >> 5;
            const uint32_t wr0 = store0 + l32s * YROW32 + 8 * khs;
            const int rsub = lane_s >> 2, c16 = lane_s & 3;
            const uint32_t rd0 = store0 + rsub * YROW32 + c16 * 16;
            uint16_t* const yl = yw + (int64_t)rsub * ldy + c16 * 8;
            const int64_t rows_left = M - mw - rsub;                   // this lane stores rows rsub + 16 it + 32 c
            auto cvt_write = [&](auto CC, auto NIC) {
                constexpr int c = decltype(CC)::value, ni = decltype(NIC)::value;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint2 o = {f2_bf16_rne(y[ni][c][4 * q + 0], y[ni][c][4 * q + 1]),
                                     f2_bf16_rne(y[ni][c][4 * q + 2], y[ni][c][4 * q + 3])};
                    lds_write8_pinned(wr0 + 16 * q, o);
                }
            };
            auto read_store = [&](auto CC, auto NIC, auto next) {
                constexpr int c = decltype(CC)::value, ni = decltype(NIC)::value;
                const uint4 v0 = lds_read16_pinned(rd0), v1 = lds_read16_pinned(rd0 + 16 * YROW32);
                next();
                if (32 * c < rows_left) *reinterpret_cast<uint4*>(yl + (int64_t)(32 * c) * ldy + ni * 32) = v0;
                if (32 * c + 16 < rows_left) *reinterpret_cast<uint4*>(yl + (int64_t)(32 * c + 16) * ldy + ni * 32) = v1;
            };
            static_assert(MT == 4, "four 32-token chunks");
            cvt_write(IC<0>{}, IC<0>{});
            read_store(IC<0>{}, IC<0>{}, [&] { cvt_write(IC<0>{}, IC<1>{}); });
            read_store(IC<0>{}, IC<1>{}, [&] { cvt_write(IC<1>{}, IC<0>{}); });
            read_store(IC<1>{}, IC<0>{}, [&] { cvt_write(IC<1>{}, IC<1>{}); });
            read_store(IC<1>{}, IC<1>{}, [&] { cvt_write(IC<2>{}, IC<0>{}); });
            read_store(IC<2>{}, IC<0>{}, [&] { cvt_write(IC<2>{}, IC<1>{}); });
            read_store(IC<2>{}, IC<1>{}, [&] { cvt_write(IC<3>{}, IC<0>{}); });
            read_store(IC<3>{}, IC<0>{}, [&] { cvt_write(IC<3>{}, IC<1>{}); });
            read_store(IC<3>{}, IC<1>{}, [] {});
        }
        if (nid < 0) break;
        id = nid;
        T = T1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // nothing may still be writing this block's LDS when it ends
}

}  // namespace

size_t packed_weight_mx_bytes(int N, int K) { return mx_wfrag_bytes(N, K) + mx_wscale_bytes(N, K); }

hipError_t launch_pack_weight_mx(const uint8_t* qw, const uint8_t* sw, int N, int K, void* out, hipStream_t stream) {
    hipLaunchKernelGGL(pack_weight_mx_kernel, dim3(1024), dim3(256), 0, stream, qw, sw, N, K, (uint8_t*)out);
    return hipGetLastError();
}

template <bool GELU>
static hipError_t launch_quantize_mx_any(const void* x, int64_t ldx, const float* inv_lambda, float rho,
                                         const void* l1p, int64_t M, int K, int r,
                                         uint8_t* qx, uint8_t* sxe, float* h, hipStream_t stream) {
    const unsigned blocks = (unsigned)((M + QROWS - 1) / QROWS);
    size_t lds = (size_t)K * sizeof(float);
    if (lds < (size_t)QHPART_BYTES) lds = QHPART_BYTES;
    if (l1p)
        hipLaunchKernelGGL((quantize_mx_kernel<true, GELU>), dim3(blocks), dim3(256), lds, stream,
                           (const uint16_t*)x, ldx, inv_lambda, rho, (const uint4*)l1p, M, K, r, qx, (uint16_t*)sxe, h);
    else
        hipLaunchKernelGGL((quantize_mx_kernel<false, GELU>), dim3(blocks), dim3(256), lds, stream,
                           (const uint16_t*)x, ldx, inv_lambda, rho, (const uint4*)nullptr, M, K, r, qx, (uint16_t*)sxe, h);
    return hipGetLastError();
}

hipError_t launch_quantize_mx(const void* x, int64_t ldx, const float* inv_lambda, float rho,
                              const void* l1p, int64_t M, int K, int r,
                              uint8_t* qx, uint8_t* sxe, float* h, bool gelu, hipStream_t stream) {
    return gelu ? launch_quantize_mx_any<true>(x, ldx, inv_lambda, rho, l1p, M, K, r, qx, sxe, h, stream)
                : launch_quantize_mx_any<false>(x, ldx, inv_lambda, rho, l1p, M, K, r, qx, sxe, h, stream);
}

// compute units of the current device (256 on MI355X; fewer in a partitioned mode), cached per device
static int cu_count() {
    static std::atomic<int> cached[64];              // 0 = not asked yet; any thread may call the library
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
        cached[dev].store(n, std::memory_order_relaxed);     // racing threads store the same value
    }
    return n;
}

// the tile-walking kernel runs one block per CU (a multiple of 8 blocks, so that a block stays on one XCD's share of
// the tile order); it needs full 256-channel tiles, a K loop of at least five stages (two more than its ring), and
// pays once every block has at least two tiles
static inline int walking_blocks() { return cu_count() / 8 * 8; }
static inline bool walks_tiles(int mtiles, int N, int K) {
    return N % 256 == 0 && K >= 576 && (int64_t)mtiles * (N / 256) >= 2 * walking_blocks();
}

hipError_t launch_linear_mx(const uint8_t* qx, const uint8_t* sxe, const void* w_packed,
                            const float* h, const void* L2, const float* bias,
                            int64_t M, int N, int K, int r, void* y, int64_t ldy, int out_f32,
                            hipStream_t stream) {
    constexpr int MT = 4;
    const uint8_t* base = (const uint8_t*)w_packed;
    const uint16_t* wsc = (const uint16_t*)(base + mx_wfrag_bytes(N, K));
    const int mtiles = (int)((M + 64 * MT - 1) / (64 * MT));
    if (walks_tiles(mtiles, N, K)) {         // 256 x 256 block tiles, eight waves, one block per CU walking its tiles
        // without a low-rank branch the kernel's h transfers still run (they have no branch): give them the codes to read
        const float* hrows = (r > 0) ? h : (const float*)qx;
        hipLaunchKernelGGL((gemm_mx_persistent_kernel<MT>), dim3((unsigned)walking_blocks()), dim3(512), 0, stream,
                           qx, (const uint16_t*)sxe, (const uint4*)base, wsc, hrows, (const uint16_t*)L2, bias,
                           M, N, K, r, y, ldy, out_f32, make_tile_grid(mtiles, N / 256));
    } else if (N % 256 == 0) {               // 256 x 256 block tiles, eight waves, one block per CU and tile
        const TileGrid tg = make_tile_grid(mtiles, N / 256);
        hipLaunchKernelGGL((gemm_mx_kernel<MT, 4, MX_LAYER>), dim3((unsigned)tile_ids(tg)), dim3(512), 0, stream,
                           qx, (const uint16_t*)sxe, (const uint4*)base, wsc, h, (const uint16_t*)L2, bias,
                           M, N, K, r, y, ldy, out_f32, tg, MxNext{});
    } else {                                 // 256 x 128 block tiles, four waves, two blocks per CU
        const TileGrid tg = make_tile_grid(mtiles, N / 128);
        hipLaunchKernelGGL((gemm_mx_kernel<MT, 2, MX_LAYER>), dim3((unsigned)tile_ids(tg)), dim3(256), 0, stream,
                           qx, (const uint16_t*)sxe, (const uint4*)base, wsc, h, (const uint16_t*)L2, bias,
                           M, N, K, r, y, ldy, out_f32, tg, MxNext{});
    }
    return hipGetLastError();
}

__global__ void zero_f32_mx_kernel(float* __restrict__ p, int64_t n) {   // a kernel, not a memset (graph replays)
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i + 4 <= n) *reinterpret_cast<float4*>(p + i) = float4{0.f, 0.f, 0.f, 0.f};
    else for (int64_t j = i; j < n; ++j) p[j] = 0.f;
}

hipError_t launch_linear_mx_next(const uint8_t* qx, const uint8_t* sxe, const void* w_packed,
                                 const float* h, const void* L2, const float* bias,
                                 int64_t M, int N, int K, int r, bool gelu,
                                 const float* next_inv_lambda, float next_rho, const void* next_l1p, int next_r,
                                 uint8_t* next_qx, uint8_t* next_sxe, float* next_h, hipStream_t stream) {
    constexpr int MT = 4;
    const uint8_t* base = (const uint8_t*)w_packed;
    const uint16_t* wsc = (const uint16_t*)(base + mx_wfrag_bytes(N, K));
    const int mtiles = (int)((M + 64 * MT - 1) / (64 * MT));
    const TileGrid tg = make_tile_grid(mtiles, N / 128);
    const MxNext nx{next_inv_lambda, (const uint4*)next_l1p, next_qx, next_sxe, next_h, next_rho, next_l1p ? next_r : 0};
    if (nx.r > 0) {                                             // the tiles ADD their shares of h'
        const int64_t n = M * next_r;
        hipLaunchKernelGGL(zero_f32_mx_kernel, dim3((unsigned)((n + 1023) / 1024)), dim3(256), 0, stream, next_h, n);
    }
    auto kern = gelu ? gemm_mx_kernel<MT, 2, MX_NEXT_GELU> : gemm_mx_kernel<MT, 2, MX_NEXT>;
    hipLaunchKernelGGL(kern, dim3((unsigned)tile_ids(tg)), dim3(256), 0, stream,
                       qx, (const uint16_t*)sxe, (const uint4*)base, wsc, h, (const uint16_t*)L2, bias,
                       M, N, K, r, (void*)nullptr, (int64_t)0, 0, tg, nx);
    return hipGetLastError();
}

}  // namespace svdq
