// C ABI of the library (declared in include/svdq.h): argument validation on
// the host, architecture check, kernel launches.  No allocation, no
// synchronisation.
#include "svdq.h"

#include <atomic>
#include <cmath>
#include <cstring>

#include "svdq_kernels.h"

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// SVDQ_OK when the current device is gfx950; cached per device index.
int check_arch() {
    static std::atomic<int> cached[64];            // 0 unknown, 1 ok, 2 unsupported; any thread may call the library
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return SVDQ_ERR_HIP;
    if (dev < 0 || dev >= 64) return SVDQ_ERR_HIP;
    int state = cached[dev].load(std::memory_order_relaxed);
    if (state == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return SVDQ_ERR_HIP;
        state = (std::strncmp(prop.gcnArchName, "gfx950", 6) == 0) ? 1 : 2;
        cached[dev].store(state, std::memory_order_relaxed);      // racing threads store the same value
    }
    return state == 1 ? SVDQ_OK : SVDQ_ERR_UNSUPPORTED_ARCH;
}

inline int hip_status(hipError_t e) { return e == hipSuccess ? SVDQ_OK : SVDQ_ERR_HIP; }

inline bool rank_ok(int r) { return r == 16 || r == 32; }

}  // namespace

extern "C" {

const char* svdq_status_string(int status) {
    switch (status) {
        case SVDQ_OK: return "ok";
        case SVDQ_ERR_INVALID_ARG: return "invalid argument";
        case SVDQ_ERR_UNSUPPORTED_SHAPE: return "unsupported shape";
        case SVDQ_ERR_UNSUPPORTED_ARCH: return "unsupported GPU architecture (gfx950 required)";
        case SVDQ_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

int svdq_version(void) { return 1; }

float svdq_alpha_lookup(const float* table, int nbins, int step, int step0, int nsteps_expert) {
    if (!table || nbins <= 0 || nsteps_expert <= 0) return NAN;
    const long long rel = (long long)step - step0;
    if (rel < 0 || rel >= nsteps_expert) return NAN;
    return table[(rel * nbins) / nsteps_expert];
}

size_t svdq_packed_l1_bytes(int K) {
    if (K <= 0 || K % SVDQ_GROUP) return 0;
    return svdq::packed_l1_bytes(K);
}

int svdq_pack_lowrank_down(const void* L1_bf16, const float* inv_lambda, int K, int r,
                           void* l1_packed, void* stream) {
    if (!L1_bf16 || !inv_lambda || !l1_packed) return SVDQ_ERR_INVALID_ARG;
    if (K <= 0 || K % SVDQ_GROUP || !rank_ok(r)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(l1_packed)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_pack_l1(L1_bf16, inv_lambda, K, r, l1_packed, (hipStream_t)stream));
}

static int quantize_nibble(const void* x_bf16, int64_t ldx, const float* inv_lambda, float rho,
                           const void* l1_packed, int64_t M, int K, int r,
                           uint8_t* qx, float* sx, float* h, bool gelu, void* stream) {
    if (!x_bf16 || !inv_lambda || !qx || !sx || M < 0) return SVDQ_ERR_INVALID_ARG;
    if (!(rho > 0.0f) || !(rho <= 1.0f)) return SVDQ_ERR_INVALID_ARG;      // also rejects NaN
    if (l1_packed ? (!h) : (r != 0)) return SVDQ_ERR_INVALID_ARG;
    if (K <= 0 || K % SVDQ_GROUP || K > SVDQ_MAX_K || ldx < K || ldx % 8) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (l1_packed && !rank_ok(r)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(x_bf16) || !aligned16(inv_lambda) || !aligned16(qx) || !aligned16(sx) ||
        !aligned16(l1_packed) || (l1_packed && !aligned16(h)))
        return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M > SVDQ_MAX_M) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M == 0) return SVDQ_OK;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_quantize(x_bf16, ldx, inv_lambda, rho, l1_packed, M, K, r, qx, sx, h, gelu,
                                            (hipStream_t)stream));
}

int svdq_quantize_act(const void* x_bf16, int64_t ldx, const float* inv_lambda, float rho,
                      const void* l1_packed, int64_t M, int K, int r,
                      uint8_t* qx, float* sx, float* h, void* stream) {
    return quantize_nibble(x_bf16, ldx, inv_lambda, rho, l1_packed, M, K, r, qx, sx, h, false, stream);
}

size_t svdq_packed_weight_bytes(int N, int K) {
    if (N <= 0 || K <= 0 || K % SVDQ_GROUP || N % SVDQ_N_TILE) return 0;
    return svdq::packed_weight_bytes(N, K);
}

int svdq_pack_weight(const uint8_t* qw, const float* sw, int N, int K, void* w_packed, void* stream) {
    if (!qw || !sw || !w_packed) return SVDQ_ERR_INVALID_ARG;
    if (N <= 0 || K <= 0 || K % SVDQ_GROUP || N % SVDQ_N_TILE) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(qw) || !aligned16(sw) || !aligned16(w_packed)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_pack_weight(qw, sw, N, K, w_packed, (hipStream_t)stream));
}

int svdq_linear_w4a4(const uint8_t* qx, const float* sx, const void* w_packed,
                     const float* h, const void* L2_bf16, const float* bias,
                     int64_t M, int N, int K, int r,
                     void* y, int64_t ldy, int out_dtype, void* stream) {
    if (!qx || !sx || !w_packed || !y || M < 0) return SVDQ_ERR_INVALID_ARG;
    if (out_dtype != SVDQ_OUT_BF16 && out_dtype != SVDQ_OUT_F32) return SVDQ_ERR_INVALID_ARG;
    if (r == 0 ? (h || L2_bf16) : (!h || !L2_bf16)) return SVDQ_ERR_INVALID_ARG;
    if (N <= 0 || K <= 0 || K % SVDQ_GROUP || N % SVDQ_N_TILE || ldy < N || ldy % 8)
        return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (r != 0 && !rank_ok(r)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(qx) || !aligned16(sx) || !aligned16(w_packed) || !aligned16(h) || !aligned16(L2_bf16) ||
        !aligned16(bias) || !aligned16(y))
        return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M > SVDQ_MAX_M) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M == 0) return SVDQ_OK;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_linear(qx, sx, w_packed, h, L2_bf16, bias, M, N, K, r, y, ldy,
                                          out_dtype == SVDQ_OUT_F32, (hipStream_t)stream));
}

int svdq_lowrank(int mode, const void* x_bf16, int64_t ldx, const float* inv_lambda,
                 const void* L_bf16, int64_t M, int K, int N, int r,
                 float* h, void* y_bf16, int64_t ldy, void* stream) {
    if (mode != 0 && mode != 1) return SVDQ_ERR_INVALID_ARG;
    if (!L_bf16 || !h || M < 0) return SVDQ_ERR_INVALID_ARG;
    if (!rank_ok(r)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (mode == 0) {
        if (!x_bf16 || !inv_lambda) return SVDQ_ERR_INVALID_ARG;
        if (K <= 0 || ldx < K) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    } else {
        if (!y_bf16) return SVDQ_ERR_INVALID_ARG;
        if (N <= 0 || ldy < N) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    }
    if (M > SVDQ_MAX_M) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M == 0) return SVDQ_OK;
    if (int a = check_arch()) return a;
    if (mode == 0)
        return hip_status(svdq::launch_lowrank_down(x_bf16, ldx, inv_lambda, L_bf16, M, K, r, h, (hipStream_t)stream));
    return hip_status(svdq::launch_lowrank_up(h, L_bf16, M, N, r, y_bf16, ldy, (hipStream_t)stream));
}

int svdq_debug_group_acc(const uint8_t* qx, const void* w_packed, int64_t M, int N, int K,
                         int64_t m0, int mt, int32_t* acc, void* stream) {
    if (!qx || !w_packed || !acc || M < 0 || m0 < 0 || mt < 0 || m0 + mt > M) return SVDQ_ERR_INVALID_ARG;
    if (N <= 0 || K <= 0 || K % SVDQ_GROUP || N % SVDQ_N_TILE) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(qx) || !aligned16(w_packed)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M > SVDQ_MAX_M) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (mt == 0) return SVDQ_OK;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_group_acc(qx, w_packed, M, N, K, m0, mt, acc, (hipStream_t)stream));
}

size_t svdq_act_e3m2_bytes(int64_t M, int K) {
    if (M < 0 || K <= 0 || K % SVDQ_GROUP) return 0;
    return svdq::act_e3m2_bytes(M, K);
}

static int quantize_e3m2(const void* x_bf16, int64_t ldx, const float* inv_lambda, float rho,
                         const void* l1_packed, int64_t M, int K, int r,
                         uint8_t* act, float* sx, float* h, bool gelu, void* stream) {
    if (!x_bf16 || !inv_lambda || !act || M < 0) return SVDQ_ERR_INVALID_ARG;
    if (!(rho > 0.0f) || !(rho <= 1.0f)) return SVDQ_ERR_INVALID_ARG;      // also rejects NaN
    if (l1_packed ? (!h) : (r != 0)) return SVDQ_ERR_INVALID_ARG;
    if (K <= 0 || K % SVDQ_GROUP || K > SVDQ_MAX_K || ldx < K || ldx % 8) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (l1_packed && !rank_ok(r)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(x_bf16) || !aligned16(inv_lambda) || !aligned16(act) || !aligned16(sx) ||
        !aligned16(l1_packed) || (l1_packed && !aligned16(h)))
        return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M > SVDQ_MAX_M) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M == 0) return SVDQ_OK;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_quantize_e3m2(x_bf16, ldx, inv_lambda, rho, l1_packed, M, K, r, act, sx, h, gelu,
                                                 (hipStream_t)stream));
}

int svdq_quantize_act_e3m2(const void* x_bf16, int64_t ldx, const float* inv_lambda, float rho,
                           const void* l1_packed, int64_t M, int K, int r,
                           uint8_t* act, float* sx, float* h, void* stream) {
    return quantize_e3m2(x_bf16, ldx, inv_lambda, rho, l1_packed, M, K, r, act, sx, h, false, stream);
}

int svdq_unpack_act_e3m2(const uint8_t* act, int64_t M, int K, uint8_t* qx, void* stream) {
    if (!act || !qx || M < 0) return SVDQ_ERR_INVALID_ARG;
    if (K <= 0 || K % SVDQ_GROUP) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(act) || !aligned16(qx)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M > SVDQ_MAX_M) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M == 0) return SVDQ_OK;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_unpack_act_e3m2(act, M, K, qx, (hipStream_t)stream));
}

size_t svdq_packed_weight_e3m2_bytes(int N, int K) {
    if (N <= 0 || K <= 0 || K % SVDQ_GROUP || N % SVDQ_N_TILE) return 0;
    return svdq::packed_weight_e3m2_bytes(N, K);
}

int svdq_pack_weight_e3m2(const uint8_t* qw, const float* sw, int N, int K, void* w_packed, void* stream) {
    if (!qw || !sw || !w_packed) return SVDQ_ERR_INVALID_ARG;
    if (N <= 0 || K <= 0 || K % SVDQ_GROUP || N % SVDQ_N_TILE) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(qw) || !aligned16(sw) || !aligned16(w_packed)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_pack_weight_e3m2(qw, sw, N, K, w_packed, (hipStream_t)stream));
}

int svdq_linear_w4a4_e3m2(const uint8_t* act, const void* w_packed,
                          const float* h, const void* L2_bf16, const float* bias,
                          int64_t M, int N, int K, int r,
                          void* y, int64_t ldy, int out_dtype, void* stream) {
    if (!act || !w_packed || !y || M < 0) return SVDQ_ERR_INVALID_ARG;
    if (out_dtype != SVDQ_OUT_BF16 && out_dtype != SVDQ_OUT_F32) return SVDQ_ERR_INVALID_ARG;
    if (r == 0 ? (h || L2_bf16) : (!h || !L2_bf16)) return SVDQ_ERR_INVALID_ARG;
    if (N <= 0 || K <= 0 || K % SVDQ_GROUP || N % SVDQ_N_TILE || ldy < N || ldy % 8)
        return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (r != 0 && !rank_ok(r)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(act) || !aligned16(w_packed) || !aligned16(h) || !aligned16(L2_bf16) ||
        !aligned16(bias) || !aligned16(y))
        return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M > SVDQ_MAX_M) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M == 0) return SVDQ_OK;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_linear_e3m2(act, w_packed, h, L2_bf16, bias, M, N, K, r, y, ldy,
                                               out_dtype == SVDQ_OUT_F32, (hipStream_t)stream));
}

int svdq_linear_w4a4_e3m2_next(const uint8_t* act, const void* w_packed,
                               const float* h, const void* L2_bf16, const float* bias,
                               int64_t M, int N, int K, int r, int gelu,
                               const float* next_inv_lambda, float next_rho,
                               const void* next_l1_packed, int next_r,
                               uint8_t* next_act, float* next_sx, float* next_h, void* stream) {
    if (!act || !w_packed || !next_inv_lambda || !next_act || M < 0) return SVDQ_ERR_INVALID_ARG;
    if (r == 0 ? (h || L2_bf16) : (!h || !L2_bf16)) return SVDQ_ERR_INVALID_ARG;
    if (!(next_rho > 0.0f) || !(next_rho <= 1.0f)) return SVDQ_ERR_INVALID_ARG;
    if (next_l1_packed ? (!next_h) : (next_r != 0)) return SVDQ_ERR_INVALID_ARG;
    if (N <= 0 || K <= 0 || K % SVDQ_GROUP || N % SVDQ_N_TILE) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if ((r != 0 && !rank_ok(r)) || (next_l1_packed && !rank_ok(next_r))) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(act) || !aligned16(w_packed) || !aligned16(h) || !aligned16(L2_bf16) || !aligned16(bias) ||
        !aligned16(next_inv_lambda) || !aligned16(next_l1_packed) || !aligned16(next_act) || !aligned16(next_sx) ||
        (next_l1_packed && !aligned16(next_h)))
        return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M > SVDQ_MAX_M) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M == 0) return SVDQ_OK;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_linear_e3m2_next(act, w_packed, h, L2_bf16, bias, M, N, K, r, gelu != 0,
                                                    next_inv_lambda, next_rho, next_l1_packed, next_r,
                                                    next_act, next_sx, next_h, (hipStream_t)stream));
}

int svdq_debug_group_acc_e3m2(const uint8_t* act, const void* w_packed, int64_t M, int N, int K,
                              int64_t m0, int mt, int32_t* acc, void* stream) {
    if (!act || !w_packed || !acc || M < 0 || m0 < 0 || mt < 0 || m0 + mt > M) return SVDQ_ERR_INVALID_ARG;
    if (N <= 0 || K <= 0 || K % SVDQ_GROUP || N % SVDQ_N_TILE) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(act) || !aligned16(w_packed)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M > SVDQ_MAX_M) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (mt == 0) return SVDQ_OK;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_group_acc_e3m2(act, w_packed, M, N, K, m0, mt, acc, (hipStream_t)stream));
}

static int quantize_mx(const void* x_bf16, int64_t ldx, const float* inv_lambda, float rho,
                       const void* l1_packed, int64_t M, int K, int r,
                       uint8_t* qx, uint8_t* sx_e8m0, float* h, bool gelu, void* stream) {
    if (!x_bf16 || !inv_lambda || !qx || !sx_e8m0 || M < 0) return SVDQ_ERR_INVALID_ARG;
    if (!(rho > 0.0f) || !(rho <= 1.0f)) return SVDQ_ERR_INVALID_ARG;
    if (l1_packed ? (!h) : (r != 0)) return SVDQ_ERR_INVALID_ARG;
    if (K <= 0 || K % SVDQ_GROUP || K > SVDQ_MAX_K || ldx < K || ldx % 8) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (l1_packed && !rank_ok(r)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(x_bf16) || !aligned16(inv_lambda) || !aligned16(qx) || !aligned16(sx_e8m0) ||
        !aligned16(l1_packed) || (l1_packed && !aligned16(h)))
        return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M > SVDQ_MAX_M) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M == 0) return SVDQ_OK;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_quantize_mx(x_bf16, ldx, inv_lambda, rho, l1_packed, M, K, r, qx, sx_e8m0, h, gelu,
                                               (hipStream_t)stream));
}

int svdq_quantize_act_mxfp4(const void* x_bf16, int64_t ldx, const float* inv_lambda, float rho,
                            const void* l1_packed, int64_t M, int K, int r,
                            uint8_t* qx, uint8_t* sx_e8m0, float* h, void* stream) {
    return quantize_mx(x_bf16, ldx, inv_lambda, rho, l1_packed, M, K, r, qx, sx_e8m0, h, false, stream);
}

int svdq_quantize_act_gelu(int format, const void* x_bf16, int64_t ldx, const float* inv_lambda, float rho,
                           const void* l1_packed, int64_t M, int K, int r,
                           uint8_t* codes, void* scales, float* h, void* stream) {
    switch (format) {
        case SVDQ_FMT_INT4:
            return quantize_nibble(x_bf16, ldx, inv_lambda, rho, l1_packed, M, K, r, codes, (float*)scales, h, true, stream);
        case SVDQ_FMT_INT4_E3M2:
            return quantize_e3m2(x_bf16, ldx, inv_lambda, rho, l1_packed, M, K, r, codes, (float*)scales, h, true, stream);
        case SVDQ_FMT_MXFP4:
            return quantize_mx(x_bf16, ldx, inv_lambda, rho, l1_packed, M, K, r, codes, (uint8_t*)scales, h, true, stream);
        default:
            return SVDQ_ERR_INVALID_ARG;
    }
}

int svdq_debug_gelu(const void* x_bf16, int64_t n, void* out_bf16, void* stream) {
    if (!x_bf16 || !out_bf16 || n < 0) return SVDQ_ERR_INVALID_ARG;
    if (n == 0) return SVDQ_OK;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_gelu(x_bf16, n, out_bf16, (hipStream_t)stream));
}

size_t svdq_packed_weight_mxfp4_bytes(int N, int K) {
    if (N <= 0 || K <= 0 || K % SVDQ_GROUP || N % SVDQ_N_TILE) return 0;
    return svdq::packed_weight_mx_bytes(N, K);
}

int svdq_pack_weight_mxfp4(const uint8_t* qw, const uint8_t* sw_e8m0, int N, int K, void* w_packed, void* stream) {
    if (!qw || !sw_e8m0 || !w_packed) return SVDQ_ERR_INVALID_ARG;
    if (N <= 0 || K <= 0 || K % SVDQ_GROUP || N % SVDQ_N_TILE) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(qw) || !aligned16(w_packed)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_pack_weight_mx(qw, sw_e8m0, N, K, w_packed, (hipStream_t)stream));
}

int svdq_linear_mxfp4(const uint8_t* qx, const uint8_t* sx_e8m0, const void* w_packed,
                      const float* h, const void* L2_bf16, const float* bias,
                      int64_t M, int N, int K, int r,
                      void* y, int64_t ldy, int out_dtype, void* stream) {
    if (!qx || !sx_e8m0 || !w_packed || !y || M < 0) return SVDQ_ERR_INVALID_ARG;
    if (out_dtype != SVDQ_OUT_BF16 && out_dtype != SVDQ_OUT_F32) return SVDQ_ERR_INVALID_ARG;
    if (r == 0 ? (h || L2_bf16) : (!h || !L2_bf16)) return SVDQ_ERR_INVALID_ARG;
    if (N <= 0 || K <= 0 || K % SVDQ_GROUP || N % SVDQ_N_TILE || ldy < N || ldy % 8)
        return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (r != 0 && !rank_ok(r)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(qx) || !aligned16(sx_e8m0) || !aligned16(w_packed) || !aligned16(h) || !aligned16(L2_bf16) ||
        !aligned16(bias) || !aligned16(y))
        return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M > SVDQ_MAX_M) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M == 0) return SVDQ_OK;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_linear_mx(qx, sx_e8m0, w_packed, h, L2_bf16, bias, M, N, K, r, y, ldy,
                                             out_dtype == SVDQ_OUT_F32, (hipStream_t)stream));
}

int svdq_linear_mxfp4_next(const uint8_t* qx, const uint8_t* sx_e8m0, const void* w_packed,
                           const float* h, const void* L2_bf16, const float* bias,
                           int64_t M, int N, int K, int r, int gelu,
                           const float* next_inv_lambda, float next_rho,
                           const void* next_l1_packed, int next_r,
                           uint8_t* next_qx, uint8_t* next_sx_e8m0, float* next_h, void* stream) {
    if (!qx || !sx_e8m0 || !w_packed || !next_inv_lambda || !next_qx || !next_sx_e8m0 || M < 0) return SVDQ_ERR_INVALID_ARG;
    if (r == 0 ? (h || L2_bf16) : (!h || !L2_bf16)) return SVDQ_ERR_INVALID_ARG;
    if (!(next_rho > 0.0f) || !(next_rho <= 1.0f)) return SVDQ_ERR_INVALID_ARG;
    if (next_l1_packed ? (!next_h) : (next_r != 0)) return SVDQ_ERR_INVALID_ARG;
    if (N <= 0 || K <= 0 || K % SVDQ_GROUP || N % SVDQ_N_TILE) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if ((r != 0 && !rank_ok(r)) || (next_l1_packed && !rank_ok(next_r))) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(qx) || !aligned16(sx_e8m0) || !aligned16(w_packed) || !aligned16(h) || !aligned16(L2_bf16) ||
        !aligned16(bias) || !aligned16(next_inv_lambda) || !aligned16(next_l1_packed) || !aligned16(next_qx) ||
        !aligned16(next_sx_e8m0) || (next_l1_packed && !aligned16(next_h)))
        return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M > SVDQ_MAX_M) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M == 0) return SVDQ_OK;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_linear_mx_next(qx, sx_e8m0, w_packed, h, L2_bf16, bias, M, N, K, r, gelu != 0,
                                                  next_inv_lambda, next_rho, next_l1_packed, next_r,
                                                  next_qx, next_sx_e8m0, next_h, (hipStream_t)stream));
}

size_t svdq_gptq_workspace_bytes(int N, int K) {
    if (N <= 0 || K <= 0 || K % SVDQ_GROUP) return 0;
    return svdq::gptq_workspace_bytes(N, K);
}

int svdq_gptq_hessian(const void* x_bf16, int64_t ldx, const float* inv_lambda, int64_t M, int K, double* H, void* stream) {
    if (!x_bf16 || !inv_lambda || !H || M < 0) return SVDQ_ERR_INVALID_ARG;
    if (K <= 0 || K % SVDQ_GROUP || ldx < K) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M > SVDQ_MAX_M) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M == 0) return SVDQ_OK;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_gptq_hessian(x_bf16, ldx, inv_lambda, M, K, H, (hipStream_t)stream));
}

int svdq_gptq_quantize(const float* R, const double* H, double damp, int N, int K, void* workspace,
                       uint8_t* qw, float* sw, void* stream) {
    if (!R || !H || !workspace || !qw || !sw) return SVDQ_ERR_INVALID_ARG;
    if (!(damp >= 0.0)) return SVDQ_ERR_INVALID_ARG;
    if (N <= 0 || K <= 0 || K % SVDQ_GROUP) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(workspace)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_gptq_quantize(R, H, damp, N, K, workspace, qw, sw, (hipStream_t)stream));
}

size_t svdq_sq_error_workspace_bytes(void) { return (size_t)svdq::SQ_ERROR_PARTIALS * sizeof(double); }

int svdq_sq_error(const void* y_ref_bf16, int64_t ld_ref, const void* y_bf16, int64_t ldy,
                  int64_t M, int N, void* workspace, double* out, void* stream) {
    if (!y_ref_bf16 || !y_bf16 || !workspace || !out || M < 0) return SVDQ_ERR_INVALID_ARG;
    if (N <= 0 || N % 8 || ld_ref < N || ldy < N || ld_ref % 8 || ldy % 8) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(y_ref_bf16) || !aligned16(y_bf16) || !aligned16(workspace)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_sq_error(y_ref_bf16, ld_ref, y_bf16, ldy, M, N, (double*)workspace, out, false,
                                            (hipStream_t)stream));
}

int svdq_sq_error_add(const void* y_ref_bf16, int64_t ld_ref, const void* y_bf16, int64_t ldy,
                      int64_t M, int N, void* workspace, double* acc, void* stream) {
    if (!y_ref_bf16 || !y_bf16 || !workspace || !acc || M < 0) return SVDQ_ERR_INVALID_ARG;
    if (N <= 0 || N % 8 || ld_ref < N || ldy < N || ld_ref % 8 || ldy % 8) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(y_ref_bf16) || !aligned16(y_bf16) || !aligned16(workspace)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_sq_error(y_ref_bf16, ld_ref, y_bf16, ldy, M, N, (double*)workspace, acc, true,
                                            (hipStream_t)stream));
}

int svdq_argmin_rows(const double* table, int nrows, int ncols, int32_t* idx, void* stream) {
    if (!table || !idx || nrows < 0 || ncols <= 0) return SVDQ_ERR_INVALID_ARG;
    if (nrows == 0) return SVDQ_OK;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_argmin_rows(table, nrows, ncols, idx, (hipStream_t)stream));
}

int svdq_sq_error_static(const void* y_ref_bf16, int64_t ld_ref, const void* y_bf16, int64_t ldy,
                         int64_t M, int N, double* out, void* stream) {
    if (!y_ref_bf16 || !y_bf16 || !out || M < 0) return SVDQ_ERR_INVALID_ARG;
    if (N <= 0 || N % 8 || ld_ref < N || ldy < N || ld_ref % 8 || ldy % 8) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (M > SVDQ_SQ_ERROR_STATIC_MAX_ELEMENTS / N) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(y_ref_bf16) || !aligned16(y_bf16)) return SVDQ_ERR_UNSUPPORTED_SHAPE;
    if (int a = check_arch()) return a;
    return hip_status(svdq::launch_sq_error_static(y_ref_bf16, ld_ref, y_bf16, ldy, M, N, out, (hipStream_t)stream));
}

int svdq_debug_scale_chain(const float* a, float rho, int64_t n, float* s, float* inv, void* stream) {
    if (!a || !s || !inv || n < 0 || n > (int64_t)1 << 31) return SVDQ_ERR_INVALID_ARG;
    if (!(rho > 0.0f) || !(rho <= 1.0f)) return SVDQ_ERR_INVALID_ARG;
    if (n == 0) return SVDQ_OK;
    if (int e = check_arch()) return e;
    return hip_status(svdq::launch_scale_chain(a, rho, n, s, inv, (hipStream_t)stream));
}

}  // extern "C"
