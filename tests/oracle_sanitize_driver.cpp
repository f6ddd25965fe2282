// Drives every entry point of the CPU oracle on small, awkward shapes (ragged rows, strided input, one thread and
// several, null optional arguments) in exactly-sized heap buffers, for a build with AddressSanitizer and
// UndefinedBehaviorSanitizer: any read or write outside a buffer, signed overflow or misaligned access aborts.
// Values are not checked here (the pins do that); a zero exit status means every call returned 0 and stayed in bounds.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "svdq_oracle.h"

static uint32_t rng_state = 12345u;
static uint32_t rnd() { rng_state = rng_state * 1664525u + 1013904223u; return rng_state >> 8; }
static uint16_t rnd_bf16() {                       // finite bf16 in roughly [-4, 4], some zeros
    const uint32_t r = rnd();
    if ((r & 15u) == 0) return 0;
    const uint16_t sign = (r & 1u) ? 0x8000u : 0u;
    const uint16_t exp = (uint16_t)(120u + (r >> 4) % 9u);       // 2^-7 .. 2^1
    return (uint16_t)(sign | (exp << 7) | ((r >> 12) & 0x7Fu));
}
#define CHECK(call) do { if ((call) != 0) { std::fprintf(stderr, "failed: %s\n", #call); return 1; } } while (0)

static size_t sz(int64_t n) { return n > 0 ? (size_t)n : 1; }      // the oracle rejects null pointers even for M = 0

static int run(int64_t M, int K, int N, int r, int64_t ldx, int nthreads) {
    std::vector<uint16_t> x(sz(M > 0 ? (M - 1) * ldx + K : 0)), L1(sz((int64_t)K * r)), L2(sz((int64_t)r * N)), ybf(sz(M * N));
    std::vector<float> il(K), sx(sz(M * (K / 64))), sw((size_t)(K / 64) * N), bias(N), y32(sz(M * N));
    std::vector<uint8_t> qx(sz(M * (K / 2))), qw((size_t)N * (K / 2)), qxm(sz(M * (K / 2))), sxm(sz(M * (K / 32))),
        swm((size_t)(K / 32) * N);
    std::vector<double> h(sz(M * r)), y64(sz(M * N));
    std::vector<int32_t> acc(sz(M * N * (K / 64)));
    for (auto& v : x) v = rnd_bf16();
    for (auto& v : L1) v = rnd_bf16();
    for (auto& v : L2) v = rnd_bf16();
    for (auto& v : il) v = 0.5f + (float)(rnd() % 1000) / 500.0f;
    for (auto& v : sw) v = 0.001f + (float)(rnd() % 1000) / 1e5f;
    for (auto& v : bias) v = (float)(rnd() % 200) / 1e3f - 0.1f;
    for (auto& v : qw) v = (uint8_t)rnd();
    for (auto& v : swm) v = (uint8_t)(118 + rnd() % 8);
    if (M > 0 && K >= 128) for (int k = 0; k < 64; ++k) x[k] = 0;             // an all-zero group
    CHECK(svdq_oracle_quantize_act(x.data(), ldx, il.data(), 0.8f, M, K, qx.data(), sx.data(), nthreads));
    if (r) CHECK(svdq_oracle_lowrank_down(x.data(), ldx, il.data(), L1.data(), M, K, r, h.data(), nthreads));
    CHECK(svdq_oracle_group_acc(qx.data(), qw.data(), M, N, K, acc.data(), nthreads));
    CHECK(svdq_oracle_linear(qx.data(), sx.data(), qw.data(), sw.data(), r ? h.data() : nullptr, r ? L2.data() : nullptr,
                             bias.data(), M, N, K, r, y64.data(), y32.data(), ybf.data(), nthreads));
    CHECK(svdq_oracle_linear(qx.data(), sx.data(), qw.data(), sw.data(), nullptr, nullptr, nullptr, M, N, K, 0,
                             nullptr, nullptr, ybf.data(), nthreads));
    CHECK(svdq_oracle_quantize_act_mxfp4(x.data(), ldx, il.data(), 0.9f, M, K, qxm.data(), sxm.data(), nthreads));
    CHECK(svdq_oracle_linear_mxfp4(qxm.data(), sxm.data(), qw.data(), swm.data(), r ? h.data() : nullptr, r ? L2.data() : nullptr,
                                   bias.data(), M, N, K, r, y64.data(), nullptr, ybf.data(), nthreads));
    std::vector<uint16_t> g(ybf.size());
    CHECK(svdq_oracle_gelu_tanh_bf16(ybf.data(), M * N, g.data()));
    (void)svdq_oracle_sq_error(ybf.data(), g.data(), M, N);
    return 0;
}

int main() {
    const float table[3] = {0.9f, 0.8f, 0.7f};
    for (int s = -1; s <= 10; ++s) (void)svdq_oracle_alpha_lookup(table, 3, s, 0, 9);
    for (int c = 0; c < 16; ++c) (void)svdq_oracle_e2m1_value(c);
    (void)svdq_oracle_f32_to_bf16(svdq_oracle_bf16_to_f32(0x3F81));
    if (run(7, 128, 5, 16, 128, 1)) return 1;          // ragged everything, one thread
    if (run(33, 192, 12, 32, 200, 3)) return 1;        // strided rows, more rows than a thread's share divides
    if (run(1, 64, 1, 0, 64, 0)) return 1;             // a single token, no low-rank branch, all threads
    if (run(0, 64, 4, 0, 64, 2)) return 1;             // no rows at all
    std::puts("oracle sanitizer drive: ok");
    return 0;
}
