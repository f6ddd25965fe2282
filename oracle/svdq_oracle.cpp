/*
 * svdq_oracle.cpp -- plain, slow, obviously-correct CPU oracle.
 *
 * TEST INFRASTRUCTURE, NOT PRODUCT (see svdq_oracle.h).  Scalar loops, no
 * intrinsics, no blocking, no fusion.  Build with
 *   g++ -std=c++17 -O2 -ffp-contract=off -fno-fast-math -shared -fPIC -pthread
 * so that every binary32 operation below is one IEEE round-to-nearest-even
 * operation (x86-64 SSE arithmetic, default rounding mode).
 *
 * Pins (tests marked "not gpu"): grid fixed point, half-step error bound,
 * printed tie vectors, clip counts, power-of-two equivariance, integer GEMM
 * special case, full-rank reconstruction of xW+b, brute force with exact
 * rationals on tiny shapes, in-group permutation invariance.
 */
#include "svdq_oracle.h"

#include <cmath>
#include <cstring>
#include <thread>
#include <vector>

namespace {

constexpr int G = SVDQ_ORACLE_GROUP;

/* Split rows [0, M) over threads; fn(m0, m1) handles rows m0 <= m < m1. */
template <class Fn>
void for_rows(int64_t M, int nthreads, Fn fn) {
    int nt = nthreads > 0 ? nthreads : svdq_oracle_hw_threads();
    if (nt < 1) nt = 1;
    if ((int64_t)nt > M) nt = (int)(M > 0 ? M : 1);
    if (nt == 1) { fn((int64_t)0, M); return; }
    std::vector<std::thread> pool;
    int64_t per = (M + nt - 1) / nt;
    for (int t = 0; t < nt; ++t) {
        int64_t m0 = (int64_t)t * per, m1 = m0 + per < M ? m0 + per : M;
        if (m0 >= m1) break;
        pool.emplace_back([=] { fn(m0, m1); });
    }
    for (auto& th : pool) th.join();
}

/* Signed value of the 4-bit two's-complement code k of a packed row. */
inline int code_at(const uint8_t* row, int k) {
    int nib = (k & 1) ? (row[k >> 1] >> 4) : (row[k >> 1] & 0xF);
    return nib >= 8 ? nib - 16 : nib;
}

}  // namespace

extern "C" {

float svdq_oracle_bf16_to_f32(uint16_t v) {
    uint32_t bits = (uint32_t)v << 16;
    float f;
    std::memcpy(&f, &bits, 4);
    return f;
}

uint16_t svdq_oracle_f32_to_bf16(float v) {
    uint32_t bits;
    std::memcpy(&bits, &v, 4);
    if ((bits & 0x7F800000u) == 0x7F800000u && (bits & 0x007FFFFFu))
        return (uint16_t)((bits >> 16) | 0x0040u);            /* quiet NaN */
    uint32_t lsb = (bits >> 16) & 1u;                         /* ties go to even */
    bits += 0x7FFFu + lsb;
    return (uint16_t)(bits >> 16);
}

int svdq_oracle_hw_threads(void) {
    unsigned n = std::thread::hardware_concurrency();
    return n ? (int)n : 1;
}

int svdq_oracle_quantize_act(const uint16_t* x, int64_t ldx, const float* inv_lambda,
                             float rho, int64_t M, int K,
                             uint8_t* qx, float* sx, int nthreads) {
    if (!x || !inv_lambda || !qx || !sx || M < 0 || K <= 0 || K % G || ldx < K) return -1;
    if (!(rho > 0.0f) || !(rho <= 1.0f)) return -1;
    const int ng = K / G;
    const float qmax = (float)SVDQ_ORACLE_QMAX;
    const float min_normal = 1.17549435e-38f;                 /* 2^-126 */
    for_rows(M, nthreads, [=](int64_t m0, int64_t m1) {
        float xs[G];
        int   q[G];
        for (int64_t m = m0; m < m1; ++m) {
            for (int g = 0; g < ng; ++g) {
                /* eq. 5: x^ = x * (1/lambda), binary32 */
                float a = 0.0f;
                for (int i = 0; i < G; ++i) {
                    int k = g * G + i;
                    xs[i] = svdq_oracle_bf16_to_f32(x[m * ldx + k]) * inv_lambda[k];
                    float ax = std::fabs(xs[i]);
                    if (ax > a) a = ax;                       /* reference magnitude m of eq. 8 */
                }
                /* eq. 8: threshold = rho * m ; eq. 9: s = threshold / q_max */
                float thr = rho * a;
                float s = thr / qmax;
                if (!(s >= min_normal)) {                     /* zero or denormal group */
                    s = 0.0f;
                    for (int i = 0; i < G; ++i) q[i] = 0;
                } else {
                    /* eq. 3 with zero-point 0: clip(round(x^/s), q_min, q_max);
                       the quotient is taken as x^ * RN(1/s), ties to even */
                    float inv = 1.0f / s;
                    for (int i = 0; i < G; ++i) {
                        float u = xs[i] * inv;
                        float rn = std::nearbyintf(u);
                        int v = rn > 7.0f ? 7 : (rn < -8.0f ? -8 : (int)rn);
                        q[i] = v;
                    }
                }
                sx[m * ng + g] = s;
                for (int i = 0; i < G; i += 2) {
                    int k = g * G + i;
                    qx[m * (K / 2) + k / 2] = (uint8_t)((q[i] & 0xF) | ((q[i + 1] & 0xF) << 4));
                }
            }
        }
    });
    return 0;
}

int svdq_oracle_lowrank_down(const uint16_t* x, int64_t ldx, const float* inv_lambda,
                             const uint16_t* L1, int64_t M, int K, int r,
                             double* h, int nthreads) {
    if (!x || !inv_lambda || !L1 || !h || M < 0 || K <= 0 || r <= 0 || ldx < K) return -1;
    for_rows(M, nthreads, [=](int64_t m0, int64_t m1) {
        for (int64_t m = m0; m < m1; ++m) {
            for (int j = 0; j < r; ++j) h[m * r + j] = 0.0;
            for (int k = 0; k < K; ++k) {
                float xs = svdq_oracle_bf16_to_f32(x[m * ldx + k]) * inv_lambda[k];   /* eq. 5 */
                for (int j = 0; j < r; ++j)
                    h[m * r + j] += (double)xs * (double)svdq_oracle_bf16_to_f32(L1[(int64_t)k * r + j]);
            }
        }
    });
    return 0;
}

int svdq_oracle_group_acc(const uint8_t* qx, const uint8_t* qw,
                          int64_t M, int N, int K, int32_t* acc, int nthreads) {
    if (!qx || !qw || !acc || M < 0 || N <= 0 || K <= 0 || K % G) return -1;
    const int ng = K / G;
    for_rows(M, nthreads, [=](int64_t m0, int64_t m1) {
        for (int64_t m = m0; m < m1; ++m)
            for (int n = 0; n < N; ++n)
                for (int g = 0; g < ng; ++g) {
                    int32_t a = 0;
                    for (int k = g * G; k < (g + 1) * G; ++k)
                        a += code_at(qx + m * (K / 2), k) * code_at(qw + (int64_t)n * (K / 2), k);
                    acc[(m * N + n) * ng + g] = a;
                }
    });
    return 0;
}

int svdq_oracle_linear(const uint8_t* qx, const float* sx,
                       const uint8_t* qw, const float* sw,
                       const double* h, const uint16_t* L2, const float* bias,
                       int64_t M, int N, int K, int r,
                       double* y64, float* y32, uint16_t* ybf16, int nthreads) {
    if (!qx || !sx || !qw || !sw || M < 0 || N <= 0 || K <= 0 || K % G || r < 0) return -1;
    if (r > 0 && (!h || !L2)) return -1;
    const int ng = K / G;
    for_rows(M, nthreads, [=](int64_t m0, int64_t m1) {
        std::vector<int8_t> arow(K);
        for (int64_t m = m0; m < m1; ++m) {
            for (int k = 0; k < K; ++k) arow[k] = (int8_t)code_at(qx + m * (K / 2), k);
            for (int n = 0; n < N; ++n) {
                const uint8_t* wrow = qw + (int64_t)n * (K / 2);
                double y = 0.0;
                for (int g = 0; g < ng; ++g) {
                    int32_t a = 0;                                       /* 4-bit branch, one group */
                    for (int k = g * G; k < (g + 1) * G; ++k) a += (int)arow[k] * code_at(wrow, k);
                    y += (double)a * (double)sx[m * ng + g] * (double)sw[(int64_t)g * N + n];
                }
                for (int j = 0; j < r; ++j)                              /* low-rank branch of eq. 7 */
                    y += h[m * r + j] * (double)svdq_oracle_bf16_to_f32(L2[(int64_t)j * N + n]);
                if (bias) y += (double)bias[n];
                float yf = (float)y;
                if (y64) y64[m * N + n] = y;
                if (y32) y32[m * N + n] = yf;
                if (ybf16) ybf16[m * N + n] = svdq_oracle_f32_to_bf16(yf);
            }
        }
    });
    return 0;
}

/* GELU in its tanh form on bf16 values, result rounded to bf16: gelu(x) = x / (1 + exp(-z)),
 * z = 2 sqrt(2/pi) (x + 0.044715 x^3).  The paper does not define the activation of the feed-forward block; this
 * is the model's, written as a fixed sequence of binary32 operations (this file is compiled without contraction,
 * so every line below is one correctly rounded operation) that a GPU can repeat bit for bit: exp(w) by
 * w = n ln 2 + r with a two-piece ln 2, a degree-5 polynomial in r, and the exponent applied exactly. */
static float gelu_tanh_f32(float x) {
    const float u = x * x;
    const float p = std::fmaf(0.044715f, u, 1.0f);
    const float t = x * p;
    const float z = 1.5957691216057308f * t;
    float w = -z;
    w = w < -87.0f ? -87.0f : (w > 87.0f ? 87.0f : w);
    const float n = std::nearbyintf(w * 1.44269504088896341f);
    float r = std::fmaf(n, -0.693359375f, w);
    r = std::fmaf(n, 2.12194440e-4f, r);
    float q = std::fmaf(1.9875691500e-4f, r, 1.3981999507e-3f);
    q = std::fmaf(q, r, 8.3334519073e-3f);
    q = std::fmaf(q, r, 4.1665795894e-2f);
    q = std::fmaf(q, r, 1.6666665459e-1f);
    q = std::fmaf(q, r, 5.0000001201e-1f);
    const float rr = r * r;
    float e = std::fmaf(q, rr, r) + 1.0f;
    e = std::ldexp(e, (int)n);
    const float s = 1.0f + e;
    const float sig = (-z > 87.0f) ? 0.0f : 1.0f / s;      /* beyond the clamp exp(-z) overflows: the result is 0 */
    return x * sig;
}

int svdq_oracle_gelu_tanh_bf16(const uint16_t* x, int64_t n, uint16_t* out) {
    if (!x || !out || n < 0) return -1;
    for (int64_t i = 0; i < n; ++i) out[i] = svdq_oracle_f32_to_bf16(gelu_tanh_f32(svdq_oracle_bf16_to_f32(x[i])));
    return 0;
}

float svdq_oracle_alpha_lookup(const float* table, int nbins, int step, int step0, int nsteps_expert) {
    if (!table || nbins <= 0 || nsteps_expert <= 0) return NAN;
    int rel = step - step0;
    if (rel < 0 || rel >= nsteps_expert) return NAN;
    int bin = (int)(((long long)rel * nbins) / nsteps_expert);
    return table[bin];
}

double svdq_oracle_sq_error(const uint16_t* y_ref, const uint16_t* y, int64_t M, int N) {
    double s = 0.0;
    for (int64_t i = 0; i < M * (int64_t)N; ++i) {
        double d = (double)svdq_oracle_bf16_to_f32(y_ref[i]) - (double)svdq_oracle_bf16_to_f32(y[i]);
        s += d * d;
    }
    return s;
}

/* ---- MXFP4 variant ---------------------------------------------------- */

static const float kE2M1[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};

float svdq_oracle_e2m1_value(int code) {
    float v = kE2M1[code & 7];
    return (code & 8) ? -v : v;
}

/* Magnitude code (0..7) of the E2M1 value nearest to mag >= 0: ties go to the
 * even code, anything beyond the largest magnitude saturates to it. */
static int e2m1_nearest(float mag) {
    int best = 0;
    float bestd = mag;                                /* distance to code 0 */
    for (int c = 1; c < 8; ++c) {
        float d = std::fabs(mag - kE2M1[c]);
        if (d < bestd || (d == bestd && (c & 1) == 0)) { best = c; bestd = d; }
    }
    return best;
}

int svdq_oracle_quantize_act_mxfp4(const uint16_t* x, int64_t ldx, const float* inv_lambda,
                                   float rho, int64_t M, int K,
                                   uint8_t* qx, uint8_t* sx, int nthreads) {
    const int B = SVDQ_ORACLE_MX_BLOCK;
    if (!x || !inv_lambda || !qx || !sx || M < 0 || K <= 0 || K % B || ldx < K) return -1;
    if (!(rho > 0.0f) || !(rho <= 1.0f)) return -1;
    const int nb = K / B;
    for_rows(M, nthreads, [=](int64_t m0, int64_t m1) {
        float xs[SVDQ_ORACLE_MX_BLOCK];
        int   q[SVDQ_ORACLE_MX_BLOCK];
        for (int64_t m = m0; m < m1; ++m) {
            for (int b = 0; b < nb; ++b) {
                float a = 0.0f;
                for (int i = 0; i < B; ++i) {
                    int k = b * B + i;
                    xs[i] = svdq_oracle_bf16_to_f32(x[m * ldx + k]) * inv_lambda[k];   /* eq. 5 */
                    float ax = std::fabs(xs[i]);
                    if (ax > a) a = ax;
                }
                float alpha = rho * a;                                                /* eq. 8 */
                int e8 = 0;
                if (alpha >= 4.70197740e-38f) {                                       /* 2^-124 */
                    int E;                                                            /* alpha = f * 2^E, f in [0.5,1) */
                    (void)std::frexp(alpha, &E);
                    int shared = (E - 1) - 2;                                         /* floor(log2 alpha) - 2 */
                    e8 = shared + 127;
                    float X = std::ldexp(1.0f, shared);
                    for (int i = 0; i < B; ++i) {
                        float v = xs[i] / X;                                          /* exact: power of two */
                        int code = e2m1_nearest(std::fabs(v));
                        if (std::signbit(xs[i])) code |= 8;
                        q[i] = code;
                    }
                } else {
                    for (int i = 0; i < B; ++i) q[i] = 0;
                }
                sx[m * nb + b] = (uint8_t)e8;
                for (int i = 0; i < B; i += 2) {
                    int k = b * B + i;
                    qx[m * (K / 2) + k / 2] = (uint8_t)(q[i] | (q[i + 1] << 4));
                }
            }
        }
    });
    return 0;
}

int svdq_oracle_linear_mxfp4(const uint8_t* qx, const uint8_t* sx,
                             const uint8_t* qw, const uint8_t* sw,
                             const double* h, const uint16_t* L2, const float* bias,
                             int64_t M, int N, int K, int r,
                             double* y64, float* y32, uint16_t* ybf16, int nthreads) {
    const int B = SVDQ_ORACLE_MX_BLOCK;
    if (!qx || !sx || !qw || !sw || M < 0 || N <= 0 || K <= 0 || K % B || r < 0) return -1;
    if (r > 0 && (!h || !L2)) return -1;
    const int nb = K / B;
    for_rows(M, nthreads, [=](int64_t m0, int64_t m1) {
        std::vector<float> arow(K);
        for (int64_t m = m0; m < m1; ++m) {
            for (int k = 0; k < K; ++k) {
                int nib = (k & 1) ? (qx[m * (K / 2) + k / 2] >> 4) : (qx[m * (K / 2) + k / 2] & 0xF);
                arow[k] = svdq_oracle_e2m1_value(nib);
            }
            for (int n = 0; n < N; ++n) {
                const uint8_t* wrow = qw + (int64_t)n * (K / 2);
                double y = 0.0;
                for (int b = 0; b < nb; ++b) {
                    double dot = 0.0;                                    /* exact: multiples of 1/4, small */
                    for (int k = b * B; k < (b + 1) * B; ++k) {
                        int nib = (k & 1) ? (wrow[k / 2] >> 4) : (wrow[k / 2] & 0xF);
                        dot += (double)arow[k] * (double)svdq_oracle_e2m1_value(nib);
                    }
                    y += dot * std::ldexp(1.0, (int)sx[m * nb + b] - 127) * std::ldexp(1.0, (int)sw[(int64_t)b * N + n] - 127);
                }
                for (int j = 0; j < r; ++j)
                    y += h[m * r + j] * (double)svdq_oracle_bf16_to_f32(L2[(int64_t)j * N + n]);
                if (bias) y += (double)bias[n];
                float yf = (float)y;
                if (y64) y64[m * N + n] = y;
                if (y32) y32[m * N + n] = yf;
                if (ybf16) ybf16[m * N + n] = svdq_oracle_f32_to_bf16(yf);
            }
        }
    });
    return 0;
}

}  /* extern "C" */
