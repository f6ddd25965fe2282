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
// operand).  Everything the matrix cores consume reaches them through LDS: a
// three-slot ring of stages (two groups each) filled by the direct global->LDS
// loads of gfx950 (global_load_lds_dwordx4 / _dword: no registers, no VALU work,
// no ds_write), requested up to three stages ahead, so the compute path has no
// global-memory waits.  Codes of both operands stay 4-bit in LDS and are unpacked
// in registers by the wave that multiplies them; weight fragments, the bf16 pieces
// of the weight scales and the correction operands are prepacked offline in
// fragment order; activations arrive group-major from the quantise kernel, which
// is fragment order already.  Block tile 128 x 128, 4 waves of 64 x 64.
//
// The K loop is a software pipeline over 32 x 32 tiles: a step issues the matrix
// instructions of tile t, then the vector ALU folds tile t-1 (results that
// completed a step ago) and unpacks operands; LDS operands are requested one
// group ahead.  The kernel is bound by vector-ALU issue (16 FMAs + 12 unpack
// operations per tile and group against 114 clocks of matrix pipe), not by the
// matrix cores.  The output tile leaves through an LDS transpose as full
// 128-byte lines.
#include "svdq_dev.h"
#include "svdq_epilogue.h"
#include "svdq_kernels.h"
#include "svdq_lds.h"
#include "svdq_tiles.h"

namespace svdq {

namespace {

constexpr int BM = 128, BN = 128;
constexpr uint32_t MAGIC_BITS = 0x40100000u;   // 2.25f
constexpr float SX_SCALE = 16384.0f;           // 2^14 = 2^22 / 256

// One LDS ring slot = one stage = two groups of a 128 x 128 block tile (byte offsets inside the slot)
constexpr uint32_t OFF_A = 0;          // activation codes, 4-bit: [group][16-byte half of the group's 32 B][token] x 16 B
constexpr uint32_t OFF_W = 8192;       // weight fragments, 4-bit: [group][n-block][lane] x 16 B
constexpr uint32_t OFF_CFR = 16384;    // n-side operand of the correction MFMA for this pair of groups: [n-block][lane] x 16 B
constexpr uint32_t OFF_SFR = 20480;    // n-side operand of the scale-product MFMA: [group][n-block][lane] x 8 B (lanes 32..63 zero)
constexpr uint32_t OFF_SXS = 24576;    // {p, p} per token: m-side operand of the scale-product MFMA: [group][token] x 8 B
constexpr uint32_t STAGE_BYTES = 26624;
constexpr int NSLOTS = 3;

// 4-bit codes -> 16*q bytes: even codes of each byte pair (k-step 0) and odd codes (k-step 1)
__device__ __forceinline__ void unpack16(const uint4 v, int4v& lo, int4v& hi) {
    const uint32_t pk[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        lo[e] = (int)((pk[e] << 4) & 0xF0F0F0F0u);
        hi[e] = (int)(pk[e] & 0xF0F0F0F0u);
    }
}

// sizes of the packed weight regions (bytes)
__host__ __device__ inline size_t wfrag_bytes(int N, int K) { return (size_t)N * (K / 2); }
__host__ __device__ inline size_t sfrag_bytes(int N, int K) { return (size_t)(N / 32) * (K / 64) * 512; }
__host__ __device__ inline size_t cfrag_bytes(int N, int K) { return (size_t)(N / 32) * ((K / 64 + 1) / 2) * 1024; }

// DUMP = false: the layer.  DUMP = true: write the int32 group accumulators of
// rows [dm0, dm0 + dmt) instead of y.
template <bool DUMP>
__global__ __launch_bounds__(256, 2)
void gemm_kernel(const uint8_t* __restrict__ qx, const float* __restrict__ sx,
                 const uint4* __restrict__ wfrag, const uint2* __restrict__ sfrag, const uint4* __restrict__ cfrag,
                 const float* __restrict__ h, const uint16_t* __restrict__ L2, const float* __restrict__ bias,
                 int64_t M, int64_t ldm, int N, int K, int r, void* __restrict__ yout, int64_t ldy, int out_f32,
                 const TileGrid tg, int64_t dm0, int dmt, int32_t* __restrict__ dacc) {
    __shared__ __attribute__((aligned(16))) uint8_t ring[NSLOTS * STAGE_BYTES];   // slot of stage s: s % 3

    int mt, nt;                                 // XCD-aware tile order (svdq_tiles.h)
    if (!tile_of(tg, blockIdx.x, mt, nt)) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);    // scalar: everything derived from it stays in SGPRs
    const int wm = wave & 1, wn = wave >> 1;
    const int l32 = lane & 31, kh = lane >> 5;
    const int ng = K >> 6;
    const int ngp = (ng + 1) >> 1;
    const int nstages = ngp;
    const int64_t m0 = (int64_t)mt * BM;
    const int n0 = nt * BN;
    const int nbB = n0 >> 5;                                       // first 32-channel block of this tile
    const uint32_t ring0 = (uint32_t)(uintptr_t)(lds_byte*)ring;

    // ---- staging.  Per stage (two groups) every wave issues seven direct global->LDS loads: two of activation
    // codes, two of weight fragments, one of correction operands, one of weight-scale pieces (1 KB each) and one
    // of 64 raw token scales (NDMA = 4 without the scale data).  Nothing passes through registers, so the
    // only waits are this code's own vmcnt waits and a whole stage can stay in flight behind the one awaited.
    // Global addresses are a wave-uniform base plus a per-lane offset fixed for the kernel.
    constexpr int NDMA = DUMP ? 4 : 7;
    uint32_t va[2], lds_a[2], lds_w[2];        // activation chunks c = 2 wave + i -> (group j = c/4, half sp = (c/2)%2, 64-row half rh = c%2)
    int cj[2];                                 // weight chunks      c = 2 wave + i -> (group j = c/4, n-block = c%4)
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = 2 * wave + i;
        const int sp = (c >> 1) & 1, rh = c & 1;
        cj[i] = c >> 2;
        const int64_t row = m0 + rh * 64 + lane;
        va[i] = (uint32_t)(((row < M) ? row : (M - 1)) * 32 + sp * 16);
        lds_a[i] = OFF_A + ((cj[i] * 2 + sp) * BM + rh * 64) * 16;
        lds_w[i] = OFF_W + ((cj[i] * 4 + (c & 3)) * 64) * 16;
    }
    const uint32_t vl16 = lane * 16;
    const uint32_t vsf = (uint32_t)(kh * ng * 512 + l32 * 16);       // scale pieces: lanes 0..31 one n-block, 32..63 the next
    const int sfj = wave >> 1, sfp = wave & 1;                        // this wave's (group, pair of n-blocks) of the scale pieces
    // token scales: wave w owns (group xg = w / 2, tokens 64 (w % 2) + lane).  The raw binary32 values land inside
    // the LDS range that the same wave then overwrites with the expanded {p, p} entries (first quarter for the
    // first half of the tokens, last quarter for the second half), so no other wave's data is touched.
    const int xrow = tid & 127;
    const int xg = wave >> 1;
    const int64_t sxrow = (m0 + xrow < M) ? (m0 + xrow) : (M - 1);
    const uint32_t vx = (uint32_t)(sxrow * 4);
    const uint32_t raw_sx = OFF_SXS + xg * 1024 + (wave & 1) * 768;

    auto stage_issue = [&](const int s) {
        const uint32_t slot = ring0 + (uint32_t)(s % NSLOTS) * STAGE_BYTES;
        const int gj[2] = {(2 * s < ng) ? 2 * s : ng - 1, (2 * s + 1 < ng) ? 2 * s + 1 : ng - 1};   // odd tail: re-read
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            dma16(qx + (size_t)gj[cj[i]] * ldm * 32, va[i], slot + lds_a[i]);
            dma16(wfrag + ((size_t)(nbB + ((2 * wave + i) & 3)) * ng + gj[cj[i]]) * 64, vl16, slot + lds_w[i]);
        }
        if (!DUMP) {
            dma16(cfrag + ((size_t)(nbB + wave) * ngp + s) * 64, vl16, slot + OFF_CFR + wave * 1024);
            dma16(sfrag + ((size_t)(nbB + 2 * sfp) * ng + gj[sfj]) * 64, vsf, slot + OFF_SFR + (sfj * 4 + 2 * sfp) * 512);
            dma4(sx + (size_t)gj[xg] * ldm, vx, slot + raw_sx);
        }
    };
    // raw token scale of this thread's (group, token), landed in `slot` -> {p, p} operand entry
    const uint32_t wr_sx = OFF_SXS + (xg * BM + xrow) * 8;
    auto scale_expand = [&](const int s, const uint32_t slot, const bool exists = false) {
        const float sc = bits_f(lds_read4(slot + raw_sx + lane * 4));
        const uint32_t p = (exists || 2 * s + xg < ng) ? split_bf16(sc * SX_SCALE) : 0u;
        lds_write8(slot + wr_sx, uint2{p, p});
    };

    // The main loop streams: each of this wave's six transfers and its token-scale load keeps a wave-uniform
    // pointer that advances by a constant per stage (two scalar adds), instead of being re-derived from s.
    // Set to stage 3 / stage 2 here; the prologue and the last stages use the generic forms above.
    const int cjw = wave >> 1;                                        // both chunks of a wave belong to the same group
    const uint32_t vw[2] = {(uint32_t)((2 * (wave & 1) + 0) * ng * 1024) + vl16, (uint32_t)((2 * (wave & 1) + 1) * ng * 1024) + vl16};
    const uint8_t* pa = qx + (size_t)(6 + cjw) * ldm * 32;
    const uint4* pw = wfrag + ((size_t)nbB * ng + 6 + cjw) * 64;
    const uint4* pc = DUMP ? nullptr : cfrag + ((size_t)(nbB + wave) * ngp + 3) * 64;
    const uint2* ps = DUMP ? nullptr : sfrag + ((size_t)(nbB + 2 * sfp) * ng + 6 + sfj) * 64;
    const float* px = DUMP ? nullptr : sx + (size_t)(6 + xg) * ldm;
    const size_t step_a = (size_t)ldm * 64, step_x = (size_t)ldm * 2;
    auto stream_issue = [&](const uint32_t slot) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            dma16(pa, va[i], slot + lds_a[i]);
            dma16(pw, vw[i], slot + lds_w[i]);
        }
        pa += step_a;
        pw += 128;
        if (!DUMP) {
            dma16(pc, vl16, slot + OFF_CFR + wave * 1024);
            dma16(ps, vsf, slot + OFF_SFR + (sfj * 4 + 2 * sfp) * 512);
            dma4(px, vx, slot + raw_sx);
            pc += 64;
            ps += 128;
            px += step_x;
        }
    };

    // the same in three parts (3 + 2 + 2 transfers; 3 + 1 + 0 without the scale operands), for the main loop
    auto stream_issue_part = [&](const uint32_t slot, const int part) {
        if (part == 0) {
            dma16(pa, va[0], slot + lds_a[0]);
            dma16(pw, vw[0], slot + lds_w[0]);
            dma16(pa, va[1], slot + lds_a[1]);
        } else if (part == 1) {
            dma16(pw, vw[1], slot + lds_w[1]);
            if (!DUMP) dma16(pc, vl16, slot + OFF_CFR + wave * 1024);
        } else {
            if (!DUMP) {
                dma16(ps, vsf, slot + OFF_SFR + (sfj * 4 + 2 * sfp) * 512);
                dma4(px, vx, slot + raw_sx);
                pc += 64;
                ps += 128;
                px += step_x;
            }
            pa += step_a;
            pw += 128;
        }
    };

    // per-lane LDS read offsets inside a slot
    const uint32_t rd_a = OFF_A + (kh * BM + wm * 64 + l32) * 16;      // + group 4096 + mi 512
    const uint32_t rd_w = OFF_W + (wn * 2 * 64 + lane) * 16;           // + group 4096 + ni 1024
    const uint32_t rd_cn = OFF_CFR + (wn * 2 * 64 + lane) * 16;        // + ni 1024
    const uint32_t rd_sf = OFF_SFR + (wn * 2 * 64 + lane) * 8;         // + group 2048 + ni 512
    const uint32_t rd_sx = OFF_SXS + (wm * 64 + l32) * 8;              // + group 1024 + mi 256
    const uint32_t rd_cp = OFF_SXS + (kh * BM + wm * 64 + l32) * 8;    // + mi 256: lanes 0..31 group g, 32..63 group g+1

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

    // prologue: stages 0..2 requested, stage 0 landed and visible, MFMA operands of group 0 requested
    stage_issue(0);
    if (nstages > 1) stage_issue(1);
    if (nstages > 2) stage_issue(2);
    if (nstages > 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * NDMA) : "memory");
    else if (nstages > 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NDMA) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (!DUMP) scale_expand(0, ring0);
    __syncthreads();
    // ---- main loop.  One step = one 32 x 32 tile of one group: its two integer MFMAs and its scale-product
    // MFMA are issued, and while they run the vector ALU finishes the PREVIOUS tile (16 FMAs on results that
    // completed a step ago) and unpacks operands.  All LDS operands are requested one group ahead.
    uint4 xpk[2], wpk[2];                      // 4-bit MFMA operands of the next group to start
    uint2 sxs[2], sfr[2];                      // scale-product operands of the same group
#pragma unroll
    for (int mi = 0; mi < 2; ++mi) {
        xpk[mi] = lds_read16(ring0 + rd_a + mi * 512);
        if (!DUMP) sxs[mi] = lds_read8(ring0 + rd_sx + mi * 256);
    }
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
        wpk[ni] = lds_read16(ring0 + rd_w + ni * 1024);
        if (!DUMP) sfr[ni] = lds_read8(ring0 + rd_sf + ni * 512);
    }

    int16v accP = magic;                       // tile (1,1) of the previous group, not yet folded into y
    float16v SP = zero16;
    uint4 cn[2], cm[2];                        // correction operands of the current pair of groups
#pragma unroll
    for (int i = 0; i < 2; ++i) cn[i] = cm[i] = uint4{0u, 0u, 0u, 0u};

    auto fold = [&](const int16v& acc, const float16v& S, float16v& yy, const int g, const int ni, const int mi) {
        if (DUMP) {
            const int64_t m = m0 + wm * 64 + mi * 32 + l32;
            if (g >= 0 && m >= dm0 && m < dm0 + dmt && m < M) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int n = n0 + wn * 64 + ni * 32 + 8 * (i >> 2) + 4 * kh + (i & 3);
                    dacc[((m - dm0) * N + n) * ng + g] = (acc[i] - (int)MAGIC_BITS) >> 8;
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) yy[i] = __builtin_fmaf(bits_f((uint32_t)acc[i]), S[i], yy[i]);
        }
    };
    auto imma = [&](const int4v& wl, const int4v& wh, const int4v& xl, const int4v& xh) -> int16v {
        int16v acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wl, xl, magic, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wh, xh, acc, 0, 0, 0);
        // DUMP: keeps the matrix instructions out of the per-lane branch around the stores of their result, where
        // they would run after operand reloads that only the active lanes perform (they read all lanes); emits nothing
        if (DUMP) asm volatile("" ::"v"(acc));
        return acc;
    };
    auto smma = [&](const uint2& sf, const uint2& sxv) -> float16v {
        if (DUMP) return zero16;
        return __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(__builtin_bit_cast(short4v, sf), __builtin_bit_cast(short4v, sxv),
                                                        zero16, 0, 0, 0);
    };
    // y -= 2.25 * (S_g + S_{g+1}) of one tile: issued right after the first of the two groups that add it, so y
    // strays from the true partial sum by at most 2.25 * S in either direction
    auto corr = [&](float16v& yy, const uint4& cnv, const uint4& cmv) {
        if (!DUMP)
            yy = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, cnv), __builtin_bit_cast(bf16x8, cmv), yy, 0, 0, 0);
    };

    // One group (j = 0 or 1 of stage s, in slot `cur`).  FULL: stages s+1..s+3 and the next group exist, so every
    // condition below is known at compile time and the body is straight-line code.
    auto group_body = [&](const int s, const uint32_t cur, const uint32_t nxt, auto JC, auto FULLC) {
        constexpr int j = decltype(JC)::value;
        constexpr bool FULL = decltype(FULLC)::value;
        const int g = 2 * s + j;
        int4v xlo[2], xhi[2], wlo[2], whi[2];

        // step 0: tile (0,0); finishes tile (1,1) of the previous group
        unpack16(wpk[0], wlo[0], whi[0]);
        unpack16(xpk[0], xlo[0], xhi[0]);
        if (!DUMP && j == 0) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                cn[i] = lds_read16(cur + rd_cn + i * 1024);
                const uint32_t cp = lds_read4(cur + rd_cp + i * 256);
                cm[i] = uint4{cp, cp, cp, cp};
            }
        }
        int16v acc0 = imma(wlo[0], whi[0], xlo[0], xhi[0]);
        float16v S0 = smma(sfr[0], sxs[0]);
        fold(accP, SP, y[1][1], g - 1, 1, 1);
        if (j == 1) corr(y[1][1], cn[1], cm[1]);
        __builtin_amdgcn_sched_barrier(0);

        // step 1: tile (0,1).  In the second group of a stage this wave no longer reads the current slot
        // (everything was requested during the first group), so after the barrier the slot can take stage
        // s+3; and stage s+1, requested two stages ago, is made visible for the prefetch in step 3.
        unpack16(xpk[1], xlo[1], xhi[1]);
        int16v acc1 = imma(wlo[0], whi[0], xlo[1], xhi[1]);
        float16v S1 = smma(sfr[0], sxs[1]);
        if (j == 1 && (FULL || s + 1 < nstages)) {
            if (FULL || s + 2 < nstages) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NDMA) : "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if (!DUMP) scale_expand(s + 1, nxt, FULL);
            __syncthreads();
            if (FULL) stream_issue_part(cur, 0);
            else if (s + 3 < nstages) stage_issue(s + 3);
        }
        // FULL: the next group's operands are requested as their registers fall free (the packed codes once they are
        // unpacked, a scale operand after the last matrix instruction that reads it), two or four reads a step, and
        // the stage's transfer requests in three parts, instead of eight reads and seven requests in one step each
        const uint32_t src = (j == 0) ? cur : nxt;
        constexpr uint32_t oa = (j == 0) ? 4096 : 0, osx = (j == 0) ? 1024 : 0, osf = (j == 0) ? 2048 : 0;
        if (FULL) {
            xpk[0] = lds_read16(src + rd_a + oa);
            wpk[0] = lds_read16(src + rd_w + oa);
        }
        fold(acc0, S0, y[0][0], g, 0, 0);
        if (j == 0) corr(y[0][0], cn[0], cm[0]);
        __builtin_amdgcn_sched_barrier(0);

        // step 2: tile (1,0)
        unpack16(wpk[1], wlo[1], whi[1]);
        acc0 = imma(wlo[1], whi[1], xlo[0], xhi[0]);
        S0 = smma(sfr[1], sxs[0]);
        if (FULL) {
            xpk[1] = lds_read16(src + rd_a + oa + 512);
            if (!DUMP) sfr[0] = lds_read8(src + rd_sf + osf);
            if (j == 1) stream_issue_part(cur, 1);
        }
        fold(acc1, S1, y[0][1], g, 0, 1);
        if (j == 0) corr(y[0][1], cn[0], cm[1]);
        __builtin_amdgcn_sched_barrier(0);

        // step 3: tile (1,1); then the operands of the next group into the registers its MFMAs have just read
        accP = imma(wlo[1], whi[1], xlo[1], xhi[1]);
        SP = smma(sfr[1], sxs[1]);
        if (FULL) {
            wpk[1] = lds_read16(src + rd_w + oa + 1024);
            if (!DUMP) {
                sxs[0] = lds_read8(src + rd_sx + osx);
                sxs[1] = lds_read8(src + rd_sx + osx + 256);
                sfr[1] = lds_read8(src + rd_sf + osf + 512);
            }
            if (j == 1) stream_issue_part(cur, 2);
        } else if (g + 1 < ng) {
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                xpk[mi] = lds_read16(src + rd_a + oa + mi * 512);
                if (!DUMP) sxs[mi] = lds_read8(src + rd_sx + osx + mi * 256);
            }
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                wpk[ni] = lds_read16(src + rd_w + oa + ni * 1024);
                if (!DUMP) sfr[ni] = lds_read8(src + rd_sf + osf + ni * 512);
            }
        }
        fold(acc0, S0, y[1][0], g, 1, 0);
        if (j == 0) corr(y[1][0], cn[1], cm[0]);
        __builtin_amdgcn_sched_barrier(0);
    };

    uint32_t cur = ring0;                      // slot of the stage being consumed
    auto next_slot = [&](const uint32_t c) { return (c == ring0 + (NSLOTS - 1) * STAGE_BYTES) ? ring0 : c + STAGE_BYTES; };
    int s = 0;
    const int nfull = ng >> 1;                 // stages with both groups
    for (; s + 3 < nfull; ++s) {               // stages up to s + 3 are complete: no clamping, no conditions
        const uint32_t nxt = next_slot(cur);
        group_body(s, cur, nxt, IC<0>{}, IC<true>{});
        group_body(s, cur, nxt, IC<1>{}, IC<true>{});
        cur = nxt;
    }
    for (; s < nstages; ++s) {
        const uint32_t nxt = next_slot(cur);
        group_body(s, cur, nxt, IC<0>{}, IC<false>{});
        if (2 * s + 1 < ng) {
            group_body(s, cur, nxt, IC<1>{}, IC<false>{});
        } else {
            corr(y[1][1], cn[1], cm[1]);       // odd group count: the last pair's correction for the tile still pending
        }
        cur = nxt;
    }
    fold(accP, SP, y[1][1], ng - 1, 1, 1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // nothing may still be writing this block's LDS when it ends

    if (DUMP) return;

    // ---- epilogue (c): low-rank up-projection on the bf16 matrix cores, bias, store
    const int64_t mw = m0 + wm * 64;                           // first token of this wave's tile
    add_lowrank_bias<2, 2>(y, h, L2, bias, mw, n0 + wn * 64, M, N, r, lane);
    if (out_f32) {
        store_tile_f32<2, 2>(y, reinterpret_cast<float*>(yout), ldy, mw, n0 + wn * 64, M, lane);
    } else {
        __syncthreads();                                       // every wave is done with the operand ring
        store_tile_bf16<2>([&](int ni, int mi, int i) { return y[ni][mi][i]; },
                           ring0 + wave * 64 * YROW, lane,
                           reinterpret_cast<uint16_t*>(yout) + mw * ldy + n0 + wn * 64, ldy, M - mw);
    }
}

// Offline packing.  Region 1: weight fragments [N/32][K/64][64 lanes][16 B]: lane (n = lane % 32, kh = lane / 32)
// holds bytes [32 g + 16 kh, +16) of row n of the canonical codes.  Region 2: n-side operands of the
// scale-product MFMA [N/32][K/64][64 lanes][8 B]: lanes kh = 0 hold bf16 {w1, w1, w2, w2} with w1 + w2 ~ sw[g][n],
// lanes kh = 1 zeros (the upper four k slots of that MFMA stay empty).  Region 3: n-side operands of the correction MFMA [N/32][ceil(ng/2)][64][16 B]: lane
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
    const size_t n2 = (size_t)(N >> 5) * ng * 64;
    for (size_t v = t0; v < n2; v += stride) {
        const int l = (int)(v & 63);
        const size_t fr = v >> 6;
        const int g = (int)(fr % ng), nb = (int)(fr / ng);
        uint2 e = {0u, 0u};
        if (l < 32) {
            const uint32_t p = split_bf16(sw[(size_t)g * N + nb * 32 + l]);
            const uint32_t w1 = p & 0xffffu, w2 = p >> 16;
            e = uint2{w1 | (w1 << 16), w2 | (w2 << 16)};
        }
        o2[v] = e;
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


hipError_t launch_linear(const uint8_t* qx, const float* sx, const void* w_packed,
                         const float* h, const void* L2, const float* bias,
                         int64_t M, int N, int K, int r, void* y, int64_t ldy, int out_f32,
                         hipStream_t stream) {
    const int mtiles = (int)((M + BM - 1) / BM), ntiles = N / BN;
    const uint8_t* base = (const uint8_t*)w_packed;
    const uint4* wf = (const uint4*)base;
    const uint2* sf = (const uint2*)(base + wfrag_bytes(N, K));
    const uint4* cf = (const uint4*)(base + wfrag_bytes(N, K) + sfrag_bytes(N, K));
    const TileGrid tg = make_tile_grid(mtiles, ntiles);
    hipLaunchKernelGGL(gemm_kernel<false>, dim3((unsigned)tile_ids(tg)), dim3(256), 0, stream,
                       qx, sx, wf, sf, cf, h, (const uint16_t*)L2, bias, M, M, N, K, r, y, ldy, out_f32,
                       tg, (int64_t)0, 0, (int32_t*)nullptr);
    return hipGetLastError();
}

hipError_t launch_group_acc(const uint8_t* qx, const void* w_packed, int64_t M, int N, int K,
                            int64_t m0, int mt, int32_t* acc, hipStream_t stream) {
    // only the token tiles that intersect [m0, m0 + mt) are launched
    const int t0 = (int)(m0 / BM), t1 = (int)((m0 + mt + BM - 1) / BM);
    const int mtiles = t1 - t0, ntiles = N / BN;
    const int64_t off = (int64_t)t0 * BM;
    // the integer accumulators need no scales: the DUMP instantiation never reads them
    const TileGrid tg = make_tile_grid(mtiles, ntiles);
    hipLaunchKernelGGL(gemm_kernel<true>, dim3((unsigned)tile_ids(tg)), dim3(256), 0, stream,
                       qx + off * 32, (const float*)nullptr, (const uint4*)w_packed, (const uint2*)nullptr,
                       (const uint4*)nullptr, (const float*)nullptr, (const uint16_t*)nullptr,
                       (const float*)nullptr, M - off, M, N, K, 0, (void*)nullptr, (int64_t)0, 0,
                       tg, m0 - off, mt, acc);
    return hipGetLastError();
}

}  // namespace svdq
