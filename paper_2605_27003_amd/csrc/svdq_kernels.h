// Host-callable launchers of the gfx950 kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace svdq {

// svdq_quantize.hip
hipError_t launch_quantize(const void* x, int64_t ldx, const float* inv_lambda, float rho,
                           const void* l1p, int64_t M, int K, int r,
                           uint8_t* qx, float* sx, float* h, bool gelu, hipStream_t stream);
hipError_t launch_gelu(const void* x, int64_t n, void* out, hipStream_t stream);
hipError_t launch_pack_l1(const void* L1, const float* inv_lambda, int K, int r, void* out, hipStream_t stream);
hipError_t launch_scale_chain(const float* a, float rho, int64_t n, float* s, float* inv, hipStream_t stream);
inline size_t packed_l1_bytes(int K) { return (size_t)(K / 64) * 4 * 2 * 64 * 16; }

// svdq_gemm.hip
size_t packed_weight_bytes(int N, int K);
hipError_t launch_pack_weight(const uint8_t* qw, const float* sw, int N, int K, void* out, hipStream_t stream);
hipError_t launch_linear(const uint8_t* qx, const float* sx, const void* w_packed,
                         const float* h, const void* L2, const float* bias,
                         int64_t M, int N, int K, int r, void* y, int64_t ldy, int out_f32,
                         hipStream_t stream);
hipError_t launch_group_acc(const uint8_t* qx, const void* w_packed, int64_t M, int N, int K,
                            int64_t m0, int mt, int32_t* acc, hipStream_t stream);

// E3M2-container variant of the int4 path (svdq_quantize.hip, svdq_gemm_e3m2.hip).  The activation operand
// buffer holds, per 64-group, Mp = round_up(M, 4) rows of 56 bytes in three planes (see quantize_kernel).
constexpr int E3M2_ROW_BYTES = 56;
inline size_t act_e3m2_bytes(int64_t M, int K) { return (size_t)(K / 64) * (size_t)((M + 3) & ~(int64_t)3) * E3M2_ROW_BYTES; }
hipError_t launch_quantize_e3m2(const void* x, int64_t ldx, const float* inv_lambda, float rho,
                                const void* l1p, int64_t M, int K, int r,
                                uint8_t* act, float* sx, float* h, bool gelu, hipStream_t stream);
size_t packed_weight_e3m2_bytes(int N, int K);
hipError_t launch_pack_weight_e3m2(const uint8_t* qw, const float* sw, int N, int K, void* out, hipStream_t stream);
hipError_t launch_linear_e3m2(const uint8_t* act, const void* w_packed,
                              const float* h, const void* L2, const float* bias,
                              int64_t M, int N, int K, int r, void* y, int64_t ldy, int out_f32,
                              hipStream_t stream);
hipError_t launch_linear_e3m2_next(const uint8_t* act, const void* w_packed,
                                   const float* h, const void* L2, const float* bias,
                                   int64_t M, int N, int K, int r, bool gelu,
                                   const float* next_inv_lambda, float next_rho, const void* next_l1p, int next_r,
                                   uint8_t* next_act, float* next_sx, float* next_h, hipStream_t stream);
hipError_t launch_group_acc_e3m2(const uint8_t* act, const void* w_packed, int64_t M, int N, int K,
                                 int64_t m0, int mt, int32_t* acc, hipStream_t stream);
hipError_t launch_unpack_act_e3m2(const uint8_t* act, int64_t M, int K, uint8_t* qx, hipStream_t stream);

// svdq_mxfp4.hip
size_t packed_weight_mx_bytes(int N, int K);
hipError_t launch_pack_weight_mx(const uint8_t* qw, const uint8_t* sw, int N, int K, void* out, hipStream_t stream);
hipError_t launch_quantize_mx(const void* x, int64_t ldx, const float* inv_lambda, float rho,
                              const void* l1p, int64_t M, int K, int r,
                              uint8_t* qx, uint8_t* sxe, float* h, bool gelu, hipStream_t stream);
hipError_t launch_linear_mx(const uint8_t* qx, const uint8_t* sxe, const void* w_packed,
                            const float* h, const void* L2, const float* bias,
                            int64_t M, int N, int K, int r, void* y, int64_t ldy, int out_f32,
                            hipStream_t stream);
hipError_t launch_linear_mx_next(const uint8_t* qx, const uint8_t* sxe, const void* w_packed,
                                 const float* h, const void* L2, const float* bias,
                                 int64_t M, int N, int K, int r, bool gelu,
                                 const float* next_inv_lambda, float next_rho, const void* next_l1p, int next_r,
                                 uint8_t* next_qx, uint8_t* next_sxe, float* next_h, hipStream_t stream);

// svdq_search.hip
constexpr int SQ_ERROR_PARTIALS = 1024;
hipError_t launch_sq_error(const void* yref, int64_t ldr, const void* y, int64_t ldy, int64_t M, int N,
                           double* workspace, double* out, bool add, hipStream_t stream);
hipError_t launch_sq_error_static(const void* yref, int64_t ldr, const void* y, int64_t ldy, int64_t M, int N,
                                  double* out, hipStream_t stream);
hipError_t launch_argmin_rows(const double* table, int nrows, int ncols, int32_t* idx, hipStream_t stream);

// svdq_gptq.hip (offline calibration)
size_t gptq_workspace_bytes(int N, int K);
hipError_t launch_gptq_hessian(const void* x, int64_t ldx, const float* inv_lambda, int64_t M, int K, double* H,
                               hipStream_t stream);
hipError_t launch_gptq_quantize(const float* R, const double* H, double damp, int N, int K, void* workspace,
                                uint8_t* qw, float* sw, hipStream_t stream);

// svdq_lowrank.hip
hipError_t launch_lowrank_down(const void* x, int64_t ldx, const float* inv_lambda, const void* L1,
                               int64_t M, int K, int r, float* h, hipStream_t stream);
hipError_t launch_lowrank_up(const float* h, const void* L2, int64_t M, int N, int r,
                             void* y, int64_t ldy, hipStream_t stream);

}  // namespace svdq
