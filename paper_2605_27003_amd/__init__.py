"""MI355X-native W4A4 SVDQuant-style linear layer (gfx950 HIP kernels behind a C ABI).

Thin Python binding over libsvdq.so: argument marshalling only.  Every step of
the path (smoothing, absmax, int4 quantise/pack, low-rank down-projection,
int4 GEMM with per-group dequantisation, low-rank up-projection, bias, bf16
store) runs in the HIP kernels.  There is no CPU fallback: if the library is
missing or the device is not gfx950 the calls raise.
"""
from .binding import (  # noqa: F401
    SvdqError, alpha_lookup, debug_group_acc, debug_scale_chain, linear_w4a4, load_library, lowrank,
    pack_lowrank_down, pack_weight, packed_l1_bytes, packed_weight_bytes, quantize_act, version,
    to_group_major, to_token_major,
    quantize_act_mxfp4, mx_to_token_major, packed_weight_mxfp4_bytes, pack_weight_mxfp4, linear_mxfp4, linear_mxfp4_next,
    ActE3M2, act_e3m2_bytes, quantize_act_e3m2, unpack_act_e3m2, packed_weight_e3m2_bytes, pack_weight_e3m2,
    linear_w4a4_e3m2, linear_w4a4_e3m2_next, debug_group_acc_e3m2,
    FMT_INT4, FMT_INT4_E3M2, FMT_MXFP4, quantize_act_gelu, debug_gelu,
    gptq_hessian, gptq_quantize,
    sq_error, sq_error_static, search_clipping_ratios,
    W4A4Linear,
)
