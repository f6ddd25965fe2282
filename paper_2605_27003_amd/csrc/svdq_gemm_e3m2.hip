// Kernels (b)+(c), E3M2-container variant: the same W4A4 arithmetic as svdq_gemm.hip (int4 codes, one exact
// integer sum per 64-group, binary32 dequantisation, fused epilogue y = main + h L2 + bias of eq. 7 / eq. 11),
// with the codes held as 6-bit floating-point fields.
//
// gfx950 has no int4 matrix instruction.  The int8 route costs two 32x32x32 matrix instructions per tile and
// group plus the nibble -> byte unpacking on the vector ALU, and that kernel is bound by vector-ALU issue.
// E3M2 (sign, 3 exponent bits, 2 mantissa bits) represents every integer of [-8, 8] exactly, products of two
// codes and their sum over a group (|sum| <= 4096) are exact in the binary32 accumulator, and
// v_mfma_scale_f32_32x32x64_f8f6f4 takes a whole 64-group in ONE instruction at twice the int8 rate.  So with
// both operands stored as E3M2 fields (weights offline, activations by the quantise kernel) the K loop has no
// unpacking at all: per 32x32 tile and group one FP6 matrix instruction (block scales 2^0, C = 0) returns the
// exact integer sums P, one bf16 matrix instruction forms the scale products S[n][m] = sw[g,n] sx[m,g] as an
// outer product of hi+lo bf16 pieces, and the vector ALU is left with one FMA per output: y += S * P.
// The price is 6 instead of 4 bits per code in HBM and LDS.
//
// Orientation and staging as in the int4 kernel: the transposed tile D[n][m] (weights are the A operand);
// block tile 128 x 128, 4 waves of 64 x 64, two blocks per CU; everything the matrix cores consume arrives by
// direct global->LDS loads into a five-slot ring of one-group stages, requested four groups ahead.  A lane's
// 24 code bytes live in two planes (bytes 0..15 and 16..23) so that LDS reads are one 16-byte and one 8-byte
// access without bank conflicts and every transfer is a full 1 KB wave-wide load.
#include "svdq_act.h"
#include "svdq_dev.h"
#include "svdq_epilogue.h"
#include "svdq_kernels.h"
#include "svdq_lds.h"
#include "svdq_quant_dev.h"
#include "svdq_tiles.h"

namespace svdq {

namespace {

constexpr int BM = 128, BN = 128;

// One LDS ring slot = one 64-group of a 128 x 128 block tile (byte offsets inside the slot)
constexpr uint32_t OFF_A0 = 0;         // activation codes, bytes 0..15:  [half][token] x 16 B
constexpr uint32_t OFF_A1 = 4096;      // activation codes, bytes 16..23: [half][token] x 8 B
constexpr uint32_t OFF_W0 = 6144;      // weight fragments, bytes 0..15:  [n-block][lane] x 16 B
constexpr uint32_t OFF_W1 = 10240;     // weight fragments, bytes 16..23: [n-block][lane] x 8 B
constexpr uint32_t OFF_SFR = 12288;    // n-side operand of the scale-product MFMA: [n-block][channel] x 8 B
constexpr uint32_t OFF_SXP = 13312;    // m-side operand: [token] x 8 B
constexpr uint32_t OFF_ZERO = 14336;   // 512 B of zeros, written once per block: the scale-product operands of k half 1
constexpr uint32_t STAGE_BYTES = 14848;
constexpr int NSLOTS = 5;

typedef int int8v __attribute__((ext_vector_type(8)));

// sizes of the packed weight regions (bytes)
__host__ __device__ inline size_t w0_bytes(int N, int K) { return (size_t)N * (K / 64) * 32; }
__host__ __device__ inline size_t w1_bytes(int N, int K) { return (size_t)N * (K / 64) * 16; }
__host__ __device__ inline size_t sf_bytes(int N, int K) { return (size_t)N * (K / 64) * 8; }

// E3M2 field of an int4 code: 0 -> 0; |q| = 2^e (1 + m/4) -> (e + 3) << 2 | m; sign in bit 5
__host__ __device__ inline uint32_t e3m2_of_code(int q) {
    const uint32_t a = (uint32_t)(q < 0 ? -q : q);
    const uint32_t t = (a == 0) ? 0u : (a == 1) ? 12u : (a < 4) ? 12u + 2u * a : (a < 8) ? 16u + a : 24u;
    return t | (q < 0 ? 32u : 0u);
}
// and back (fields produced by the above only)
__device__ __forceinline__ int code_of_e3m2(uint32_t f) {
    const uint32_t t = f & 31u;
    const int a = (t == 0) ? 0 : (t == 12) ? 1 : (t < 20) ? (int)(t - 12) / 2 : (t < 24) ? (int)t - 16 : 8;
    return (f & 32u) ? -a : a;
}

// One wave-wide 16-byte transfer stream: a wave-uniform base that advances by `stride` bytes per group, a
// per-lane byte offset and a destination inside the slot, all fixed for the kernel.
struct Stream {
    const uint8_t* base;
    size_t stride;
    uint32_t voff;
    uint32_t lds;
};

// What the kernel does with the finished tile.
//   MODE_LAYER      store y (bf16 or binary32): the layer.
//   MODE_DUMP       test hook: write the integer group sums of rows [dm0, dm0 + dmt) instead of y.
//   MODE_NEXT       y never reaches HBM: the wave rounds its 64 x 64 tile to bf16 (what MODE_LAYER would have
//   MODE_NEXT_GELU  stored), optionally applies GELU, and runs the NEXT layer's quantise pass on it: a wave's 64
//                   channels are exactly one 64-group of the next layer's K axis, so it writes that group's block
//                   of the next activation operand buffer (codes, scale pieces, optionally sx) and adds its share
//                   of the next low-rank projection h' = x^' L1' to the (zeroed) binary32 h' with atomic adds.
enum { MODE_LAYER = 0, MODE_DUMP = 1, MODE_NEXT = 2, MODE_NEXT_GELU = 3 };

// The next layer's side of MODE_NEXT*: smoothing vector [N], clipping ratio, packed L1' (pack_l1_kernel order,
// K' = N) and rank, outputs.
struct NextLayer {
    const float* inv_lambda;
    const uint4* l1p;
    uint8_t* act;
    float* sx;
    float* h;
    float rho;
    int r;
};

template <int MODE>
__global__ __launch_bounds__(256, 2)
void gemm_e3m2_kernel(const uint8_t* __restrict__ act, const uint8_t* __restrict__ w0, const uint8_t* __restrict__ w1,
                      const uint8_t* __restrict__ sfr,
                      const float* __restrict__ h, const uint16_t* __restrict__ L2, const float* __restrict__ bias,
                      int64_t M, int N, int K, int r, void* __restrict__ yout, int64_t ldy, int out_f32,
                      int tile0, const TileGrid tg, int64_t dm0, int dmt, int32_t* __restrict__ dacc,
                      const NextLayer nx) {
    constexpr bool DUMP = MODE == MODE_DUMP, NEXT = MODE >= MODE_NEXT, GELU = MODE == MODE_NEXT_GELU;
    __shared__ __attribute__((aligned(16))) uint8_t ring[NSLOTS * STAGE_BYTES];   // slot of group g: g % 5

    int mt, nt;                                 // XCD-aware tile order (svdq_tiles.h)
    if (!tile_of(tg, blockIdx.x, mt, nt)) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int l32 = lane & 31, kh = lane >> 5;
    const int ng = K >> 6;
    const int64_t Mp = (M + 3) & ~(int64_t)3;
    const int64_t m0 = (int64_t)(tile0 + mt) * BM;
    const int n0 = nt * BN;
    const int nbB = n0 >> 5;
    const uint32_t ring0 = (uint32_t)(uintptr_t)(lds_byte*)ring;

    // ---- staging.  Per group the block needs 4 + 2 KB of activation codes, 4 + 2 KB of weight codes, 1 KB of
    // weight-scale pieces and 1 KB of token-scale pieces: every wave issues four 1 KB transfers (three without
    // scales).  Stream 0: bytes 0..15 of the activation fragments of (half wave / 2, tokens 64 (wave % 2) + lane).
    // Stream 1: bytes 0..15 of the weight fragments of n-block `wave`.  Stream 2: the 8-byte planes, activations
    // of half `wave` on waves 0, 1 (a lane moves two tokens), weights of n-blocks 2 (wave - 2) + {0, 1} on waves
    // 2, 3.  Stream 3: the weight-scale pieces of all four n-blocks on even waves, the token-scale pieces on odd
    // waves (a lane moves two tokens).  Waves 2, 3 repeat what waves 0, 1 move
    // there, so that every wave counts the same number of transfers and the loop has no wave-dependent branch.
    constexpr int NDMA = DUMP ? 3 : 4;
    const size_t gstride = (size_t)Mp * E3M2_ROW_BYTES;
    Stream st[4];
    {
        const int64_t row = m0 + (wave & 1) * 64 + lane;
        st[0] = Stream{act, gstride, (uint32_t)(((row < M) ? row : (M - 1)) * 32 + (wave >> 1) * 16),
                       OFF_A0 + (uint32_t)((wave >> 1) * BM + (wave & 1) * 64) * 16};
        st[1] = Stream{w0 + (size_t)nbB * ng * 1024, 1024, (uint32_t)(wave * ng * 1024 + lane * 16), OFF_W0 + (uint32_t)wave * 1024};
        const int64_t pr = (m0 + 2 * lane < Mp - 2) ? (m0 + 2 * lane) : (Mp - 2);
        if (wave < 2) {
            st[2] = Stream{act + (size_t)Mp * 32 + (size_t)wave * Mp * 8, gstride, (uint32_t)(pr * 8), OFF_A1 + (uint32_t)wave * 1024};
        } else {
            st[2] = Stream{w1 + (size_t)(nbB + 2 * (wave - 2)) * ng * 512, 512, (uint32_t)(kh * ng * 512 + l32 * 16),
                           OFF_W1 + (uint32_t)(wave - 2) * 1024};
        }
        if (DUMP) {
            st[3] = st[2];
        } else if ((wave & 1) == 0) {
            st[3] = Stream{sfr + (size_t)nbB * ng * 256, 256, (uint32_t)((lane >> 4) * ng * 256 + (lane & 15) * 16), OFF_SFR};
        } else {
            st[3] = Stream{act + (size_t)Mp * 48, gstride, (uint32_t)(pr * 8), OFF_SXP};
        }
    }
    auto stage_issue = [&](const int g) {
        const uint32_t slot = ring0 + (uint32_t)(g % NSLOTS) * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < NDMA; ++i) dma16(st[i].base + (size_t)g * st[i].stride, st[i].voff, slot + st[i].lds);
    };
    // The main loop streams: the four transfers keep wave-uniform pointers that advance by a constant per group.
    const uint8_t* sp[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) sp[i] = st[i].base + (size_t)4 * st[i].stride;      // first streamed group: 4
    auto stream_issue = [&](const uint32_t slot) {
#pragma unroll
        for (int i = 0; i < NDMA; ++i) {
            dma16(sp[i], st[i].voff, slot + st[i].lds);
            sp[i] += st[i].stride;
        }
    };

    // per-lane LDS read offsets inside a slot
    const uint32_t rd_x0 = OFF_A0 + (uint32_t)(kh * BM + wm * 64 + l32) * 16;      // + mi 512
    const uint32_t rd_x1 = OFF_A1 + (uint32_t)(kh * BM + wm * 64 + l32) * 8;       // + mi 256
    const uint32_t rd_w0 = OFF_W0 + (uint32_t)(wn * 2 * 64 + lane) * 16;           // + ni 1024
    const uint32_t rd_w1 = OFF_W1 + (uint32_t)(wn * 2 * 64 + lane) * 8;            // + ni 512
    // The scale product needs K = 4 of the matrix instruction's 8: the lanes of k half 1 read zeros on both sides (an
    // area of every slot that no transfer touches).  Multipliers fed 0 x 0 switch nothing, which on this power-limited
    // chip is worth 1 % of the kernel's time against feeding both halves half the scale.
    const uint32_t rd_sf = kh ? OFF_ZERO + (uint32_t)l32 * 8 : OFF_SFR + (uint32_t)(wn * 2 * 32 + l32) * 8;   // + ni 256
    const uint32_t rd_sx = kh ? OFF_ZERO + (uint32_t)l32 * 8 : OFF_SXP + (uint32_t)(wm * 64 + l32) * 8;       // + mi 256
    if (!DUMP && tid < 32 * NSLOTS)                      // visible after the barrier that ends the prologue
        *reinterpret_cast<uint4*>(ring + (tid >> 5) * STAGE_BYTES + OFF_ZERO + (tid & 31) * 16) = uint4{0u, 0u, 0u, 0u};

    float16v y[2][2];                        // [ni][mi]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) y[a][b][i] = 0.0f;
    float16v zero16;
#pragma unroll
    for (int i = 0; i < 16; ++i) zero16[i] = 0.0f;

    // wait until at most k groups' worth of this wave's transfers are outstanding
    auto wait_groups = [&](const int k) {
        if (k <= 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        else if (k == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NDMA) : "memory");
        else if (k == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * NDMA) : "memory");
        else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(3 * NDMA) : "memory");
    };
    // prologue: groups 0..3 requested; while they are in flight y starts as the low-rank term plus the bias
    // (eq. 7, 11: the bf16 matrix cores form h L2 from hi+lo bf16 pieces of h), so that the latency of these loads
    // hides behind the first operand transfers instead of standing at the end of the tile; then group 0 is
    // awaited and made visible.
    const int pre = ng < NSLOTS - 1 ? ng : NSLOTS - 1;
    for (int g = 0; g < pre; ++g) stage_issue(g);
    if (!DUMP) add_lowrank_bias<2, 2>(y, h, L2, bias, m0 + wm * 64, n0 + wn * 64, M, N, r, lane);
    wait_groups(pre - 1);
    __syncthreads();

    // MFMA operands of one group: code fragments (24 B per lane) and scale pieces.  Two register sets: a group's
    // operands are requested from LDS as soon as its slot is visible (right after the barrier in the group
    // before), a good three tile steps ahead of their first use, into the set the current group is not using.
    struct Operands {
        uint4 xlo[2], wlo[2];
        uint2 xhi[2], whi[2], sf[2], sxp[2];
    };
    Operands op0, op1;
    auto fetch = [&](Operands& o, const uint32_t slot) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
            o.xlo[mi] = lds_read16(slot + rd_x0 + mi * 512);
            o.xhi[mi] = lds_read8_pinned(slot + rd_x1 + mi * 256);
            if (!DUMP) o.sxp[mi] = lds_read8(slot + rd_sx + mi * 256);
        }
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            o.wlo[ni] = lds_read16(slot + rd_w0 + ni * 1024);
            o.whi[ni] = lds_read8_pinned(slot + rd_w1 + ni * 512);
            if (!DUMP) o.sf[ni] = lds_read8(slot + rd_sf + ni * 256);
        }
    };
    // the same in four parts, for the loop: the token side and the channel side of tile block hf
    auto fetch_x = [&](Operands& o, const uint32_t slot, const int hf) {
        o.xlo[hf] = lds_read16_pinned(slot + rd_x0 + hf * 512);
        o.xhi[hf] = lds_read8_pinned(slot + rd_x1 + hf * 256);
        if (!DUMP) o.sxp[hf] = lds_read8_pinned(slot + rd_sx + hf * 256);
    };
    auto fetch_w = [&](Operands& o, const uint32_t slot, const int hf) {
        o.wlo[hf] = lds_read16_pinned(slot + rd_w0 + hf * 1024);
        o.whi[hf] = lds_read8_pinned(slot + rd_w1 + hf * 512);
        if (!DUMP) o.sf[hf] = lds_read8_pinned(slot + rd_sf + hf * 256);
    };
    auto stream_issue_part = [&](const uint32_t slot, const int i0, const int i1) {
#pragma unroll
        for (int i = i0; i < i1; ++i)
            if (i < NDMA) {
                dma16(sp[i], st[i].voff, slot + st[i].lds);
                sp[i] += st[i].stride;
            }
    };
    fetch(op0, ring0);

    // exact integer sums of one tile and group: E3M2 x E3M2, block scales 2^0 (E8M0 127), C = 0
    auto pmma = [&](const Operands& o, const int ni, const int mi) -> float16v {
        const int8v a = {(int)o.wlo[ni].x, (int)o.wlo[ni].y, (int)o.wlo[ni].z, (int)o.wlo[ni].w, (int)o.whi[ni].x, (int)o.whi[ni].y, 0, 0};
        const int8v b = {(int)o.xlo[mi].x, (int)o.xlo[mi].y, (int)o.xlo[mi].z, (int)o.xlo[mi].w, (int)o.xhi[mi].x, (int)o.xhi[mi].y, 0, 0};
        return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, zero16, 3, 3, 0, 0x7f, 0, 0x7f);
    };
    // S[n][m] = sw[n] sx[m]: n side {w1, w1, w2, w2}, m side {x1, x2, x1, x2} in k half 0, zeros in k half 1
    auto smma = [&](const Operands& o, const int ni, const int mi) -> float16v {
        if (DUMP) return zero16;
        return __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(__builtin_bit_cast(short4v, o.sf[ni]),
                                                        __builtin_bit_cast(short4v, o.sxp[mi]), zero16, 0, 0, 0);
    };
    auto fold = [&](const float16v& P, const float16v& S, float16v& yy, const int g, const int ni, const int mi) {
        if (DUMP) {
            const int64_t m = m0 + wm * 64 + mi * 32 + l32;
            if (g >= 0 && m >= dm0 && m < dm0 + dmt && m < M) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int n = n0 + wn * 64 + ni * 32 + 8 * (i >> 2) + 4 * kh + (i & 3);
                    dacc[((m - dm0) * N + n) * ng + g] = (int32_t)P[i];
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) yy[i] = __builtin_fmaf(P[i], S[i], yy[i]);
            // keeps the tile a contiguous register tuple inside the loop (the epilogue's matrix instructions need
            // one); without it the 16 values are allocated separately and re-assembled by copies in every iteration
            asm volatile("" : "+v"(yy));
        }
    };

    // Two (P, S) register sets alternate between the four tiles of a group: set A takes tiles (0,0) and (1,0),
    // set B tiles (0,1) and (1,1); a set is folded into y one step after its matrix instructions were issued.
    float16v PA, SA, PB = zero16, SB = zero16;  // B: tile (1,1) of the previous group, not yet folded into y

    // Matrix instructions have no side effects, so the compiler places them wherever it likes inside a basic block
    // and scheduling fences do not hold them.  This empty statement "reads" their results, which fixes the issue
    // point of a tile's two instructions; it also passes the accumulator tile that the following fold updates, so that
    // fold cannot be placed ahead of them.  It emits nothing.
    // In the DUMP instantiation it keeps the matrix instruction out of the per-lane branch around the stores of
    // its result: sunk into that branch it would run after operand reloads that only the active lanes perform
    // (the instruction itself reads all lanes).
    auto issued = [&](const float16v& P, const float16v& S, float16v& ynext) {
        if (DUMP) asm volatile("" ::"v"(P));
        else asm volatile("" : "+v"(ynext) : "v"(P), "v"(S));
    };

    // One group in slot `cur`, operands in `o`; the next group's go to `on`.  A step issues the two matrix
    // instructions of one tile and, while they run, the vector ALU folds the previous tile.  FULL: groups
    // g+1..g+4 exist, so the body is straight-line code.
    auto group_body = [&](const int g, const uint32_t cur, const uint32_t nxt, auto SETC, auto FULLC) {
        constexpr bool FULL = decltype(FULLC)::value;
        constexpr int SET = decltype(SETC)::value;
        const Operands& o = SET ? op1 : op0;
        Operands& on = SET ? op0 : op1;
        const uint32_t prev = (cur == ring0) ? ring0 + (NSLOTS - 1) * STAGE_BYTES : cur - STAGE_BYTES;
        // step 0: tile (0,0); finishes tile (1,1) of the previous group.  Every wave took its operands of this group
        // from `cur` a group ago, so the previous group's slot can take group g + 4.  The next group's twelve LDS
        // reads and the four transfer requests are spread over the four steps (three reads and one request each):
        // as one run of sixteen memory instructions in a single step they cost 5 % of the kernel.
        PA = pmma(o, 0, 0);
        SA = smma(o, 0, 0);
        issued(PA, SA, y[1][1]);
        if (FULL) {
            // One barrier per PAIR of groups (operand set 0 = even group g): it waits until only group g + 3 is in
            // flight, so groups g + 1 and g + 2, whose operands are read during g and g + 1, are visible to all
            // waves; and every wave has finished its reads of slots g - 1 and g (issued during g - 2 and g - 1),
            // which take groups g + 4 and g + 5 during this pair.
            if (SET == 0) {
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NDMA) : "memory");
                __syncthreads();
            }
            fetch_x(on, nxt, 0);
            stream_issue_part(prev, 0, 1);
        }
        fold(PB, SB, y[1][1], g - 1, 1, 1);
        __builtin_amdgcn_sched_barrier(0);

        // step 1: tile (0,1)
        PB = pmma(o, 0, 1);
        SB = smma(o, 0, 1);
        issued(PB, SB, y[0][0]);
        if (FULL) {
            fetch_w(on, nxt, 0);
            stream_issue_part(prev, 1, 2);
        } else if (g + 1 < ng) {
            wait_groups((ng - 1 < g + 3 ? ng - 1 : g + 3) - (g + 1));
            __syncthreads();
            if (g + 4 < ng) stage_issue(g + 4);
            fetch(on, nxt);
        }
        fold(PA, SA, y[0][0], g, 0, 0);
        __builtin_amdgcn_sched_barrier(0);

        // step 2: tile (1,0)
        PA = pmma(o, 1, 0);
        SA = smma(o, 1, 0);
        issued(PA, SA, y[0][1]);
        if (FULL) {
            fetch_x(on, nxt, 1);
            stream_issue_part(prev, 2, 3);
        }
        fold(PB, SB, y[0][1], g, 0, 1);
        __builtin_amdgcn_sched_barrier(0);

        // step 3: tile (1,1)
        PB = pmma(o, 1, 1);
        SB = smma(o, 1, 1);
        issued(PB, SB, y[1][0]);
        if (FULL) {
            fetch_w(on, nxt, 1);
            stream_issue_part(prev, 3, 4);
        }
        fold(PA, SA, y[1][0], g, 1, 0);
        __builtin_amdgcn_sched_barrier(0);
    };

    // Main loop, ten groups per iteration (the five ring slots times the two operand sets): slot addresses are
    // compile-time constants there, so they ride in the offset fields of the LDS instructions instead of costing
    // vector-ALU additions per group.
    auto slot_of = [&](const int i) { return ring0 + (uint32_t)(i % NSLOTS) * STAGE_BYTES; };
    int g = 0;
    for (; g + 13 < ng; g += 10) {
        group_body(g + 0, slot_of(0), slot_of(1), IC<0>{}, IC<1>{});
        group_body(g + 1, slot_of(1), slot_of(2), IC<1>{}, IC<1>{});
        group_body(g + 2, slot_of(2), slot_of(3), IC<0>{}, IC<1>{});
        group_body(g + 3, slot_of(3), slot_of(4), IC<1>{}, IC<1>{});
        group_body(g + 4, slot_of(4), slot_of(0), IC<0>{}, IC<1>{});
        group_body(g + 5, slot_of(0), slot_of(1), IC<1>{}, IC<1>{});
        group_body(g + 6, slot_of(1), slot_of(2), IC<0>{}, IC<1>{});
        group_body(g + 7, slot_of(2), slot_of(3), IC<1>{}, IC<1>{});
        group_body(g + 8, slot_of(3), slot_of(4), IC<0>{}, IC<1>{});
        group_body(g + 9, slot_of(4), slot_of(0), IC<1>{}, IC<1>{});
    }
    // the rest with run-time slot addresses: complete pairs first, then the last groups with their conditions
    uint32_t cur = ring0;                      // g is a multiple of ten here
    auto next_slot = [&](const uint32_t c) { return (c == ring0 + (NSLOTS - 1) * STAGE_BYTES) ? ring0 : c + STAGE_BYTES; };
    for (; g + 5 < ng; g += 2) {               // two groups per iteration: the operand sets swap roles without copies
        const uint32_t nxt = next_slot(cur), nx2 = next_slot(nxt);
        group_body(g, cur, nxt, IC<0>{}, IC<1>{});
        group_body(g + 1, nxt, nx2, IC<1>{}, IC<1>{});
        cur = nx2;
    }
    for (; g < ng; g += 2) {
        const uint32_t nxt = next_slot(cur), nx2 = next_slot(nxt);
        group_body(g, cur, nxt, IC<0>{}, IC<0>{});
        if (g + 1 < ng) group_body(g + 1, nxt, nx2, IC<1>{}, IC<0>{});
        cur = nx2;
    }
    fold(PB, SB, y[1][1], ng - 1, 1, 1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // nothing may still be writing this block's LDS when it ends

    if (DUMP) return;

    const int64_t mw = m0 + wm * 64;                           // first token of this wave's tile
    if constexpr (NEXT) {
        // ---- the next layer's kernel (a) on this wave's tile.  Lane (l32, kh) holds, of token mw + 32 mi + l32,
        // channels 32 ni + 8 q + 4 kh + j (register 4 q + j of y[ni][mi]).  After rounding (and GELU) the values
        // are packed in pairs and the lanes l, l + 32 trade n-blocks: lane kh keeps the 32 consecutive channels
        // 32 kh .. 32 kh + 31 of its token, which is the lane layout of the quantise kernel (and the A operand of
        // the bf16 matrix instruction that forms h').
        const int gq = (n0 + wn * 64) >> 6;                    // this wave's group of the next layer
        const float* il = nx.inv_lambda + n0 + wn * 64 + kh * 32;
        uint4 bfrag[4][2];
        if (nx.r > 0) {
            const uint4* pb = nx.l1p + (size_t)gq * (4 * 2 * 64) + lane;
#pragma unroll
            for (int sI = 0; sI < 4; ++sI) {
                bfrag[sI][0] = pb[(sI * 2 + 0) * 64];
                bfrag[sI][1] = pb[(sI * 2 + 1) * 64];
            }
        }
        uint8_t* blk = nx.act + (size_t)gq * Mp * E3M2_ROW_BYTES;
        float16v hp[2];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
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
                xc[q] = uint4{e0[0], e1[0], e0[1], e1[1]};     // channels 32 kh + 8 q + 0..7
            }
            LaneCodes<true> codes;
            float sc;
            quantize_rows<true>(xc, il, nx.rho, codes, sc);
            const int64_t row = mw + mi * 32 + l32;
            if (row < M) {
                *reinterpret_cast<uint4*>(blk + (size_t)row * 32 + kh * 16) = codes.lo;
                *reinterpret_cast<uint2*>(blk + (size_t)Mp * 32 + ((size_t)kh * Mp + row) * 8) = codes.hi;
                if (kh == 0) {
                    const uint32_t p = split_bf16(sc);
                    *reinterpret_cast<uint2*>(blk + (size_t)Mp * 48 + (size_t)row * 8) = uint2{p, p};
                    if (nx.sx) nx.sx[(size_t)gq * M + row] = sc;
                }
            }
            if (nx.r > 0) {
                hp[mi] = zero16;                               // [token][j]: lane holds column j = l32
#pragma unroll
                for (int sI = 0; sI < 4; ++sI) {
                    const bf16x8 av = __builtin_bit_cast(bf16x8, xc[sI]);
                    hp[mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8, bfrag[sI][0]), hp[mi], 0, 0, 0);
                    hp[mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8, bfrag[sI][1]), hp[mi], 0, 0, 0);
                }
            }
        }
        if (nx.r > 0) {
            // the two waves that share tokens (wn = 0, 1) add their shares in LDS first: half the atomic adds
            __syncthreads();                                   // every wave is done with the operand ring
            float* part = reinterpret_cast<float*>(ring) + wm * (2 * 16 * 64) + lane;
            if (wn == 1) {
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int i = 0; i < 16; ++i) part[(mi * 16 + i) * 64] = hp[mi][i];
            }
            __syncthreads();
            if (wn == 0) {
                float tot[2][16];                              // all LDS reads first: one wait, not one per add
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int i = 0; i < 16; ++i) tot[mi][i] = hp[mi][i] + part[(mi * 16 + i) * 64];
                // register (mi, i) is token mw + 4 kh + [32 mi + 8 (i / 4) + i % 4] of column l32
                const int64_t first = mw + 4 * kh;
                const int left = (l32 < nx.r && first < M) ? (int)((M - first < 64) ? M - first : 64) : 0;
                float* hb = nx.h + first * nx.r + l32;
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int rl = 32 * mi + 8 * (i >> 2) + (i & 3);
                        if (rl < left) unsafeAtomicAdd(hb + rl * nx.r, tot[mi][i]);
                    }
            }
        }
        return;
    }

    // ---- epilogue (c): store (the low-rank term and the bias are already in y)
    if (out_f32) {
        store_tile_f32<2, 2>(y, reinterpret_cast<float*>(yout), ldy, mw, n0 + wn * 64, M, lane);
    } else {
        __syncthreads();                                       // every wave is done with the operand ring
        store_tile_bf16<2>([&](int ni, int mi, int i) { return y[ni][mi][i]; },
                           ring0 + wave * 64 * YROW, lane,
                           reinterpret_cast<uint16_t*>(yout) + mw * ldy + n0 + wn * 64, ldy, M - mw);
    }
}

// Offline packing from the canonical form (qw [N][K/2] nibbles, sw [K/64][N] binary32).
// Region 1: bytes 0..15 of the weight fragments, [N/32][K/64][64 lanes][16 B]; region 2: bytes 16..23,
// [N/32][K/64][64 lanes][8 B]: lane (n = lane % 32, kh = lane / 32) holds the E3M2 fields of k = 64 g + 32 kh + 0..31
// of channel n, k ascending from bit 0.  Region 3: n-side operands of the scale-product MFMA,
// [N/32][K/64][32 channels][8 B]: bf16 {w1, w1, w2, w2} with w1 + w2 ~ sw[g][n] (the lanes of k half 0 read the
// entry; those of k half 1 read zeros).
__global__ void pack_weight_e3m2_kernel(const uint8_t* __restrict__ qw, const float* __restrict__ sw,
                                        int N, int K, uint8_t* __restrict__ out) {
    const int ng = K >> 6;
    const size_t stride = (size_t)gridDim.x * blockDim.x, t0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint4* o1 = reinterpret_cast<uint4*>(out);
    uint2* o2 = reinterpret_cast<uint2*>(out + w0_bytes(N, K));
    const size_t n1 = (size_t)(N >> 5) * ng * 64;
    for (size_t v = t0; v < n1; v += stride) {
        const int lane = (int)(v & 63);
        const size_t fr = v >> 6;
        const int g = (int)(fr % ng), nb = (int)(fr / ng);
        const int n = nb * 32 + (lane & 31), kh = lane >> 5;
        const uint4 nib = *reinterpret_cast<const uint4*>(qw + (size_t)n * (K >> 1) + g * 32 + kh * 16);
        const uint32_t nw[4] = {nib.x, nib.y, nib.z, nib.w};
        uint32_t f[6] = {0u, 0u, 0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            const int q = (int)((nw[j >> 3] >> (4 * (j & 7))) & 15u);
            const uint64_t fld = (uint64_t)e3m2_of_code(q >= 8 ? q - 16 : q) << ((6 * j) & 31);
            f[(6 * j) >> 5] |= (uint32_t)fld;
            if (((6 * j) & 31) > 26) f[((6 * j) >> 5) + 1] |= (uint32_t)(fld >> 32);
        }
        o1[v] = uint4{f[0], f[1], f[2], f[3]};
        o2[v] = uint2{f[4], f[5]};
    }
    uint2* o3 = reinterpret_cast<uint2*>(out + w0_bytes(N, K) + w1_bytes(N, K));
    const size_t n3 = (size_t)(N >> 5) * ng * 32;
    for (size_t v = t0; v < n3; v += stride) {
        const int l = (int)(v & 31);
        const size_t fr = v >> 5;
        const int g = (int)(fr % ng), nb = (int)(fr / ng);
        const uint32_t p = split_bf16(sw[(size_t)g * N + nb * 32 + l]);
        const uint32_t w1 = p & 0xffffu, w2 = p >> 16;
        o3[v] = uint2{w1 | (w1 << 16), w2 | (w2 << 16)};
    }
}

// Activation operand buffer -> nibble codes qx [K/64][M][32 B] (the layout of the int4 path)
__global__ void unpack_act_e3m2_kernel(const uint8_t* __restrict__ act, int64_t M, int K, uint8_t* __restrict__ qx) {
    const int ng = K >> 6;
    const int64_t Mp = (M + 3) & ~(int64_t)3;
    const int64_t total = (int64_t)ng * M * 2;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < total; v += (int64_t)gridDim.x * blockDim.x) {
        const int hf = (int)(v & 1);
        const int64_t row = (v >> 1) % M;
        const int g = (int)((v >> 1) / M);
        const uint8_t* blk = act + (size_t)g * Mp * E3M2_ROW_BYTES;
        const uint4 lo = *reinterpret_cast<const uint4*>(blk + (size_t)row * 32 + hf * 16);
        const uint2 hi = *reinterpret_cast<const uint2*>(blk + (size_t)Mp * 32 + ((size_t)hf * Mp + row) * 8);
        const uint32_t f[7] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, 0u};
        uint32_t nw[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            const int bit = 6 * j;
            const uint64_t two = (uint64_t)f[bit >> 5] | ((uint64_t)f[(bit >> 5) + 1] << 32);
            const int q = code_of_e3m2((uint32_t)(two >> (bit & 31)) & 63u);
            nw[j >> 3] |= (uint32_t)(q & 15) << (4 * (j & 7));
        }
        *reinterpret_cast<uint4*>(qx + ((size_t)g * M + row) * 32 + hf * 16) = uint4{nw[0], nw[1], nw[2], nw[3]};
    }
}

// h' of the emitting modes starts at zero.  A kernel, not a memset: memset nodes misbehave in replayed graphs.
__global__ void zero_f32_kernel(float* __restrict__ p, int64_t n) {
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i + 4 <= n) *reinterpret_cast<float4*>(p + i) = float4{0.f, 0.f, 0.f, 0.f};
    else for (int64_t j = i; j < n; ++j) p[j] = 0.f;
}


}  // namespace

size_t packed_weight_e3m2_bytes(int N, int K) { return w0_bytes(N, K) + w1_bytes(N, K) + sf_bytes(N, K); }

hipError_t launch_pack_weight_e3m2(const uint8_t* qw, const float* sw, int N, int K, void* out, hipStream_t stream) {
    hipLaunchKernelGGL(pack_weight_e3m2_kernel, dim3(1024), dim3(256), 0, stream, qw, sw, N, K, (uint8_t*)out);
    return hipGetLastError();
}

hipError_t launch_unpack_act_e3m2(const uint8_t* act, int64_t M, int K, uint8_t* qx, hipStream_t stream) {
    hipLaunchKernelGGL(unpack_act_e3m2_kernel, dim3(1024), dim3(256), 0, stream, act, M, K, qx);
    return hipGetLastError();
}

hipError_t launch_linear_e3m2(const uint8_t* act, const void* w_packed,
                              const float* h, const void* L2, const float* bias,
                              int64_t M, int N, int K, int r, void* y, int64_t ldy, int out_f32,
                              hipStream_t stream) {
    const int mtiles = (int)((M + BM - 1) / BM), ntiles = N / BN;
    const uint8_t* base = (const uint8_t*)w_packed;
    const TileGrid tg = make_tile_grid(mtiles, ntiles);
    hipLaunchKernelGGL(gemm_e3m2_kernel<MODE_LAYER>, dim3((unsigned)tile_ids(tg)), dim3(256), 0, stream,
                       act, base, base + w0_bytes(N, K), base + w0_bytes(N, K) + w1_bytes(N, K),
                       h, (const uint16_t*)L2, bias, M, N, K, r, y, ldy, out_f32,
                       0, tg, (int64_t)0, 0, (int32_t*)nullptr, NextLayer{});
    return hipGetLastError();
}

hipError_t launch_linear_e3m2_next(const uint8_t* act, const void* w_packed,
                                   const float* h, const void* L2, const float* bias,
                                   int64_t M, int N, int K, int r, bool gelu,
                                   const float* next_inv_lambda, float next_rho, const void* next_l1p, int next_r,
                                   uint8_t* next_act, float* next_sx, float* next_h, hipStream_t stream) {
    const int mtiles = (int)((M + BM - 1) / BM), ntiles = N / BN;
    const uint8_t* base = (const uint8_t*)w_packed;
    const NextLayer nx{next_inv_lambda, (const uint4*)next_l1p, next_act, next_sx, next_h, next_rho, next_l1p ? next_r : 0};
    if (nx.r > 0) {                                             // the tiles ADD their shares of h'
        const int64_t n = M * next_r;
        hipLaunchKernelGGL(zero_f32_kernel, dim3((unsigned)((n + 1023) / 1024)), dim3(256), 0, stream, next_h, n);
    }
    auto kern = gelu ? gemm_e3m2_kernel<MODE_NEXT_GELU> : gemm_e3m2_kernel<MODE_NEXT>;
    const TileGrid tg = make_tile_grid(mtiles, ntiles);
    hipLaunchKernelGGL(kern, dim3((unsigned)tile_ids(tg)), dim3(256), 0, stream,
                       act, base, base + w0_bytes(N, K), base + w0_bytes(N, K) + w1_bytes(N, K),
                       h, (const uint16_t*)L2, bias, M, N, K, r, (void*)nullptr, (int64_t)0, 0,
                       0, tg, (int64_t)0, 0, (int32_t*)nullptr, nx);
    return hipGetLastError();
}

hipError_t launch_group_acc_e3m2(const uint8_t* act, const void* w_packed, int64_t M, int N, int K,
                                 int64_t m0, int mt, int32_t* acc, hipStream_t stream) {
    // only the token tiles that intersect [m0, m0 + mt) are launched
    const int t0 = (int)(m0 / BM), t1 = (int)((m0 + mt + BM - 1) / BM);
    const int mtiles = t1 - t0, ntiles = N / BN;
    const uint8_t* base = (const uint8_t*)w_packed;
    const TileGrid tg = make_tile_grid(mtiles, ntiles);
    hipLaunchKernelGGL(gemm_e3m2_kernel<MODE_DUMP>, dim3((unsigned)tile_ids(tg)), dim3(256), 0, stream,
                       act, base, base + w0_bytes(N, K), (const uint8_t*)nullptr,
                       (const float*)nullptr, (const uint16_t*)nullptr, (const float*)nullptr,
                       M, N, K, 0, (void*)nullptr, (int64_t)0, 0,
                       t0, tg, m0, mt, acc, NextLayer{});
    return hipGetLastError();
}

}  // namespace svdq
