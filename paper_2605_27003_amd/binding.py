"""ctypes binding of include/svdq.h for torch tensors (device memory and streams only)."""
import collections
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsvdq.so")
_lib = None

OUT_BF16, OUT_F32 = 0, 1
_vp, _i64, _i32, _f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float

EXPORTS = {
    "svdq_status_string": (ctypes.c_char_p, [_i32]),
    "svdq_version": (_i32, []),
    "svdq_alpha_lookup": (_f32, [_vp, _i32, _i32, _i32, _i32]),
    "svdq_packed_l1_bytes": (ctypes.c_size_t, [_i32]),
    "svdq_pack_lowrank_down": (_i32, [_vp, _vp, _i32, _i32, _vp, _vp]),
    "svdq_quantize_act": (_i32, [_vp, _i64, _vp, _f32, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp]),
    "svdq_packed_weight_bytes": (ctypes.c_size_t, [_i32, _i32]),
    "svdq_pack_weight": (_i32, [_vp, _vp, _i32, _i32, _vp, _vp]),
    "svdq_linear_w4a4": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _i64, _i32, _i32, _i32, _vp, _i64, _i32, _vp]),
    "svdq_lowrank": (_i32, [_i32, _vp, _i64, _vp, _vp, _i64, _i32, _i32, _i32, _vp, _vp, _i64, _vp]),
    "svdq_act_e3m2_bytes": (ctypes.c_size_t, [_i64, _i32]),
    "svdq_quantize_act_e3m2": (_i32, [_vp, _i64, _vp, _f32, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp]),
    "svdq_unpack_act_e3m2": (_i32, [_vp, _i64, _i32, _vp, _vp]),
    "svdq_packed_weight_e3m2_bytes": (ctypes.c_size_t, [_i32, _i32]),
    "svdq_pack_weight_e3m2": (_i32, [_vp, _vp, _i32, _i32, _vp, _vp]),
    "svdq_linear_w4a4_e3m2": (_i32, [_vp, _vp, _vp, _vp, _vp, _i64, _i32, _i32, _i32, _vp, _i64, _i32, _vp]),
    "svdq_linear_w4a4_e3m2_next": (_i32, [_vp, _vp, _vp, _vp, _vp, _i64, _i32, _i32, _i32, _i32,
                                          _vp, _f32, _vp, _i32, _vp, _vp, _vp, _vp]),
    "svdq_debug_group_acc_e3m2": (_i32, [_vp, _vp, _i64, _i32, _i32, _i64, _i32, _vp, _vp]),
    "svdq_quantize_act_gelu": (_i32, [_i32, _vp, _i64, _vp, _f32, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp]),
    "svdq_debug_gelu": (_i32, [_vp, _i64, _vp, _vp]),
    "svdq_quantize_act_mxfp4": (_i32, [_vp, _i64, _vp, _f32, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp]),
    "svdq_packed_weight_mxfp4_bytes": (ctypes.c_size_t, [_i32, _i32]),
    "svdq_pack_weight_mxfp4": (_i32, [_vp, _vp, _i32, _i32, _vp, _vp]),
    "svdq_linear_mxfp4": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _i64, _i32, _i32, _i32, _vp, _i64, _i32, _vp]),
    "svdq_linear_mxfp4_next": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _i64, _i32, _i32, _i32, _i32,
                                      _vp, _f32, _vp, _i32, _vp, _vp, _vp, _vp]),
    "svdq_gptq_workspace_bytes": (ctypes.c_size_t, [_i32, _i32]),
    "svdq_gptq_hessian": (_i32, [_vp, _i64, _vp, _i64, _i32, _vp, _vp]),
    "svdq_gptq_quantize": (_i32, [_vp, _vp, ctypes.c_double, _i32, _i32, _vp, _vp, _vp, _vp]),
    "svdq_sq_error_workspace_bytes": (ctypes.c_size_t, []),
    "svdq_sq_error": (_i32, [_vp, _i64, _vp, _i64, _i64, _i32, _vp, _vp, _vp]),
    "svdq_sq_error_add": (_i32, [_vp, _i64, _vp, _i64, _i64, _i32, _vp, _vp, _vp]),
    "svdq_argmin_rows": (_i32, [_vp, _i32, _i32, _vp, _vp]),
    "svdq_sq_error_static": (_i32, [_vp, _i64, _vp, _i64, _i64, _i32, _vp, _vp]),
    "svdq_debug_group_acc": (_i32, [_vp, _vp, _i64, _i32, _i32, _i64, _i32, _vp, _vp]),
    "svdq_debug_scale_chain": (_i32, [_vp, _f32, _i64, _vp, _vp, _vp]),
}


class SvdqError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {load_library().svdq_status_string(status).decode()} ({status})")


def load_library(build_if_missing=True):
    """Load libsvdq.so (built in-tree by paper_2605_27003_amd/build.py); never falls back to anything else."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            if not build_if_missing:
                raise FileNotFoundError(_LIB_PATH)
            from . import build as _build
            _build.build(force=True)
        lib = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc, where):
    if rc != 0:
        raise SvdqError(rc, where)


def version():
    return int(load_library().svdq_version())


def alpha_lookup(table, step, step0, nsteps_expert):
    arr = (ctypes.c_float * len(table))(*table)
    return float(load_library().svdq_alpha_lookup(ctypes.cast(arr, _vp), len(table), step, step0, nsteps_expert))


def packed_l1_bytes(K):
    return int(load_library().svdq_packed_l1_bytes(K))


def packed_weight_bytes(N, K):
    return int(load_library().svdq_packed_weight_bytes(N, K))


def pack_lowrank_down(L1_bf16, inv_lambda):
    """L1 [K,r] bf16, inv_lambda [K] f32 (device) -> opaque uint8 tensor for quantize_act."""
    K, r = L1_bf16.shape
    out = torch.empty(packed_l1_bytes(K), dtype=torch.uint8, device=L1_bf16.device)
    _check(load_library().svdq_pack_lowrank_down(_ptr(L1_bf16), _ptr(inv_lambda), K, r, _ptr(out), _stream()),
           "svdq_pack_lowrank_down")
    return out


def pack_weight(qw, sw):
    """qw [N,K/2] uint8 canonical codes, sw [K/64,N] f32 (device) -> opaque uint8 tensor for linear_w4a4."""
    N, K2 = qw.shape
    K = 2 * K2
    out = torch.empty(packed_weight_bytes(N, K), dtype=torch.uint8, device=qw.device)
    _check(load_library().svdq_pack_weight(_ptr(qw), _ptr(sw), N, K, _ptr(out), _stream()), "svdq_pack_weight")
    return out


def quantize_act(x_bf16, inv_lambda, rho, l1_packed=None, r=0, out=None):
    """x [M,K] bf16 (row stride allowed) -> (qx [K/64,M,32] u8, sx [K/64,M] f32, h [M,r] f32 or None).

    qx and sx are group-major (see include/svdq.h); `to_token_major` gives the [M,K/2] / [M,K/64] view."""
    M, K = x_bf16.shape
    assert x_bf16.dtype == torch.bfloat16 and x_bf16.stride(1) == 1
    dev = x_bf16.device
    if out is None:
        qx = torch.empty((K // 64, M, 32), dtype=torch.uint8, device=dev)
        sx = torch.empty((K // 64, M), dtype=torch.float32, device=dev)
        h = torch.empty((M, r), dtype=torch.float32, device=dev) if l1_packed is not None else None
    else:
        qx, sx, h = out
    ldx = x_bf16.stride(0) if M > 1 else K
    _check(load_library().svdq_quantize_act(_ptr(x_bf16), ldx, _ptr(inv_lambda), float(rho), _ptr(l1_packed),
                                           M, K, r if l1_packed is not None else 0,
                                           _ptr(qx), _ptr(sx), _ptr(h), _stream()), "svdq_quantize_act")
    return qx, sx, h


def to_token_major(qx, sx):
    """Group-major (qx [K/64,M,32], sx [K/64,M]) -> token-major copies (qx [M,K/2], sx [M,K/64])."""
    ng, M, _ = qx.shape
    return qx.permute(1, 0, 2).reshape(M, ng * 32).contiguous(), sx.t().contiguous()


def to_group_major(qx_tm, sx_tm):
    """Token-major (qx [M,K/2], sx [M,K/64]) -> group-major copies, the layout the GEMM consumes."""
    M, K2 = qx_tm.shape
    return qx_tm.reshape(M, K2 // 32, 32).permute(1, 0, 2).contiguous(), sx_tm.t().contiguous()


def linear_w4a4(qx, sx, w_packed, N, h=None, L2_bf16=None, bias=None, out=None, out_dtype=torch.bfloat16):
    """qx [K/64,M,32], sx [K/64,M] (group-major) -> y [M,N] bf16 (or f32: the value before the bf16 rounding)."""
    ng, M, _ = qx.shape
    K = 64 * ng
    r = 0 if h is None else h.shape[1]
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=qx.device)
    code = OUT_F32 if out.dtype == torch.float32 else OUT_BF16
    ldy = out.stride(0) if M > 1 else N
    _check(load_library().svdq_linear_w4a4(_ptr(qx), _ptr(sx), _ptr(w_packed), _ptr(h), _ptr(L2_bf16), _ptr(bias),
                                          M, N, K, r, _ptr(out), ldy, code, _stream()), "svdq_linear_w4a4")
    return out


def lowrank(mode, *, x_bf16=None, inv_lambda=None, L_bf16=None, h=None, y_bf16=None):
    """mode 0: h = (x*inv_lambda) L1 (returns h); mode 1: y += h L2 in place (returns y)."""
    lib = load_library()
    if mode == 0:
        M, K = x_bf16.shape
        r = L_bf16.shape[1]
        if h is None:
            h = torch.empty((M, r), dtype=torch.float32, device=x_bf16.device)
        ldx = x_bf16.stride(0) if M > 1 else K
        _check(lib.svdq_lowrank(0, _ptr(x_bf16), ldx, _ptr(inv_lambda), _ptr(L_bf16), M, K, 0, r,
                                _ptr(h), None, 0, _stream()), "svdq_lowrank")
        return h
    M, N = y_bf16.shape
    r = L_bf16.shape[0]
    ldy = y_bf16.stride(0) if M > 1 else N
    _check(lib.svdq_lowrank(1, None, 0, None, _ptr(L_bf16), M, 0, N, r, _ptr(h), _ptr(y_bf16), ldy, _stream()),
           "svdq_lowrank")
    return y_bf16


def debug_group_acc(qx, w_packed, N, m0, mt):
    """int32 group accumulators of rows [m0, m0+mt) as the GEMM kernel forms them -> [mt, N, K/64]."""
    ng, M, _ = qx.shape
    K = 64 * ng
    acc = torch.empty((mt, N, K // 64), dtype=torch.int32, device=qx.device)
    _check(load_library().svdq_debug_group_acc(_ptr(qx), _ptr(w_packed), M, N, K, m0, mt, _ptr(acc), _stream()),
           "svdq_debug_group_acc")
    return acc


# ---- E3M2-container execution of the int4 layer -------------------------------------------------
class ActE3M2(collections.namedtuple("ActE3M2", "buf M K")):
    """Activation operand buffer of the FP6 matrix-core path (layout in include/svdq.h) with its logical shape."""


def act_e3m2_bytes(M, K):
    return load_library().svdq_act_e3m2_bytes(M, K)


def quantize_act_e3m2(x_bf16, inv_lambda, rho, l1_packed=None, r=0, out=None, want_sx=True):
    """x [M,K] bf16 -> (act ActE3M2, sx [K/64,M] f32 or None, h [M,r] f32 or None).  Same codes and scales as
    quantize_act, codes held as E3M2 fields."""
    M, K = x_bf16.shape
    assert x_bf16.dtype == torch.bfloat16 and x_bf16.stride(1) == 1
    dev = x_bf16.device
    if out is None:
        act = ActE3M2(torch.empty(act_e3m2_bytes(M, K), dtype=torch.uint8, device=dev), M, K)
        sx = torch.empty((K // 64, M), dtype=torch.float32, device=dev) if want_sx else None
        h = torch.empty((M, r), dtype=torch.float32, device=dev) if l1_packed is not None else None
    else:
        act, sx, h = out
        assert act.M == M and act.K == K
    ldx = x_bf16.stride(0) if M > 1 else K
    _check(load_library().svdq_quantize_act_e3m2(_ptr(x_bf16), ldx, _ptr(inv_lambda), float(rho), _ptr(l1_packed),
                                                M, K, r if l1_packed is not None else 0,
                                                _ptr(act.buf), _ptr(sx), _ptr(h), _stream()), "svdq_quantize_act_e3m2")
    return act, sx, h


def unpack_act_e3m2(act):
    """ActE3M2 -> nibble codes qx [K/64,M,32] u8 in the layout of quantize_act."""
    qx = torch.empty((act.K // 64, act.M, 32), dtype=torch.uint8, device=act.buf.device)
    _check(load_library().svdq_unpack_act_e3m2(_ptr(act.buf), act.M, act.K, _ptr(qx), _stream()), "svdq_unpack_act_e3m2")
    return qx


def packed_weight_e3m2_bytes(N, K):
    return load_library().svdq_packed_weight_e3m2_bytes(N, K)


def pack_weight_e3m2(qw, sw, out=None):
    """qw [N,K/2] uint8 canonical codes, sw [K/64,N] f32 (device) -> opaque uint8 tensor for linear_w4a4_e3m2.
    `out`: a caller's buffer of at least packed_weight_e3m2_bytes(N, K) bytes (e.g. one staging buffer shared by
    every layer of a model whose weights stay resident in the canonical 4-bit form)."""
    N, K2 = qw.shape
    K = 2 * K2
    if out is None:
        out = torch.empty(packed_weight_e3m2_bytes(N, K), dtype=torch.uint8, device=qw.device)
    assert out.numel() >= packed_weight_e3m2_bytes(N, K)
    _check(load_library().svdq_pack_weight_e3m2(_ptr(qw), _ptr(sw), N, K, _ptr(out), _stream()), "svdq_pack_weight_e3m2")
    return out


def linear_w4a4_e3m2(act, w_packed, N, h=None, L2_bf16=None, bias=None, out=None, out_dtype=torch.bfloat16):
    """ActE3M2 -> y [M,N] bf16 (or f32: the value before the bf16 rounding)."""
    M, K = act.M, act.K
    r = 0 if h is None else h.shape[1]
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=act.buf.device)
    code = OUT_F32 if out.dtype == torch.float32 else OUT_BF16
    ldy = out.stride(0) if M > 1 else N
    _check(load_library().svdq_linear_w4a4_e3m2(_ptr(act.buf), _ptr(w_packed), _ptr(h), _ptr(L2_bf16), _ptr(bias),
                                               M, N, K, r, _ptr(out), ldy, code, _stream()), "svdq_linear_w4a4_e3m2")
    return out


def linear_w4a4_e3m2_next(act, w_packed, N, next_inv_lambda, next_rho, h=None, L2_bf16=None, bias=None, gelu=True,
                          next_l1_packed=None, next_r=0, out=None, want_sx=True):
    """The layer on `act` fused with the NEXT layer's quantise pass (optionally through GELU): returns what
    quantize_act_e3m2 / quantize_act_gelu(FMT_INT4_E3M2) of this layer's bf16 output would return,
    (ActE3M2 of shape [M, N], sx [N/64, M] or None, h' [M, next_r] or None), without y ever being stored."""
    M, K = act.M, act.K
    r = 0 if h is None else h.shape[1]
    dev = act.buf.device
    if out is None:
        nact = ActE3M2(torch.empty(act_e3m2_bytes(M, N), dtype=torch.uint8, device=dev), M, N)
        nsx = torch.empty((N // 64, M), dtype=torch.float32, device=dev) if want_sx else None
        nh = torch.empty((M, next_r), dtype=torch.float32, device=dev) if next_l1_packed is not None else None
    else:
        nact, nsx, nh = out
        assert nact.M == M and nact.K == N
    _check(load_library().svdq_linear_w4a4_e3m2_next(
        _ptr(act.buf), _ptr(w_packed), _ptr(h), _ptr(L2_bf16), _ptr(bias), M, N, K, r, int(bool(gelu)),
        _ptr(next_inv_lambda), float(next_rho), _ptr(next_l1_packed), next_r if next_l1_packed is not None else 0,
        _ptr(nact.buf), _ptr(nsx), _ptr(nh), _stream()), "svdq_linear_w4a4_e3m2_next")
    return nact, nsx, nh


def debug_group_acc_e3m2(act, w_packed, N, m0, mt):
    """Integer group sums of rows [m0, m0+mt) as the FP6 matrix-core path forms them -> [mt, N, K/64] int32."""
    acc = torch.empty((mt, N, act.K // 64), dtype=torch.int32, device=act.buf.device)
    _check(load_library().svdq_debug_group_acc_e3m2(_ptr(act.buf), _ptr(w_packed), act.M, N, act.K, m0, mt,
                                                   _ptr(acc), _stream()), "svdq_debug_group_acc_e3m2")
    return acc


# ---- kernel (a) with GELU fused ----------------------------------------------------------------
FMT_INT4, FMT_INT4_E3M2, FMT_MXFP4 = 0, 1, 2


def quantize_act_gelu(fmt, x_bf16, inv_lambda, rho, l1_packed=None, r=0, out=None):
    """quantize_act / quantize_act_e3m2 / quantize_act_mxfp4 (fmt = FMT_*) of gelu(x), the activation applied on the
    fly; returns what that function returns."""
    M, K = x_bf16.shape
    assert x_bf16.dtype == torch.bfloat16 and x_bf16.stride(1) == 1
    dev = x_bf16.device
    if out is None:
        h = torch.empty((M, r), dtype=torch.float32, device=dev) if l1_packed is not None else None
        if fmt == FMT_INT4_E3M2:
            codes = ActE3M2(torch.empty(act_e3m2_bytes(M, K), dtype=torch.uint8, device=dev), M, K)
            scales = torch.empty((K // 64, M), dtype=torch.float32, device=dev)
        else:
            codes = torch.empty((K // 64, M, 32), dtype=torch.uint8, device=dev)
            scales = (torch.empty((K // 64, M), dtype=torch.float32, device=dev) if fmt == FMT_INT4
                      else torch.empty(((K // 64 + 1) // 2, M, 2, 2), dtype=torch.uint8, device=dev))
    else:
        codes, scales, h = out
    buf = codes.buf if fmt == FMT_INT4_E3M2 else codes
    ldx = x_bf16.stride(0) if M > 1 else K
    _check(load_library().svdq_quantize_act_gelu(fmt, _ptr(x_bf16), ldx, _ptr(inv_lambda), float(rho), _ptr(l1_packed),
                                                M, K, r if l1_packed is not None else 0,
                                                _ptr(buf), _ptr(scales), _ptr(h), _stream()), "svdq_quantize_act_gelu")
    return codes, scales, h


def debug_gelu(x_bf16):
    """bf16 tensor -> bf16(gelu(x)) through the device function of the fused quantise pass."""
    x = x_bf16.contiguous()
    out = torch.empty_like(x)
    _check(load_library().svdq_debug_gelu(_ptr(x), x.numel(), _ptr(out), _stream()), "svdq_debug_gelu")
    return out


# ---- GPTQ on the residual (offline calibration) ------------------------------------------------
def gptq_hessian(x_bf16, inv_lambda, H=None):
    """H [K,K] f64 += X^T X^ over the rows of x (a new zero H if none is given)."""
    M, K = x_bf16.shape
    if H is None:
        H = torch.zeros((K, K), dtype=torch.float64, device=x_bf16.device)
    ldx = x_bf16.stride(0) if M > 1 else K
    _check(load_library().svdq_gptq_hessian(_ptr(x_bf16), ldx, _ptr(inv_lambda), M, K, _ptr(H), _stream()), "svdq_gptq_hessian")
    return H


def gptq_quantize(R_f32, H_f64, damp=0.01):
    """R [K,N] f32 residual, H [K,K] f64 -> (qw [N,K/2] u8 canonical codes, sw [K/64,N] f32 scales)."""
    K, N = R_f32.shape
    dev = R_f32.device
    ws = torch.empty(load_library().svdq_gptq_workspace_bytes(N, K), dtype=torch.uint8, device=dev)
    qw = torch.empty((N, K // 2), dtype=torch.uint8, device=dev)
    sw = torch.empty((K // 64, N), dtype=torch.float32, device=dev)
    _check(load_library().svdq_gptq_quantize(_ptr(R_f32.contiguous()), _ptr(H_f64.contiguous()), float(damp), N, K,
                                            _ptr(ws), _ptr(qw), _ptr(sw), _stream()), "svdq_gptq_quantize")
    return qw, sw


# ---- MXFP4 variant ---------------------------------------------------------------------------
def quantize_act_mxfp4(x_bf16, inv_lambda, rho, l1_packed=None, r=0, out=None):
    """x [M,K] bf16 -> (qx [K/64,M,32] u8 E2M1 codes, sx [ceil(K/128),M,2,2] u8 E8M0 bytes, h [M,r] f32 or None)."""
    M, K = x_bf16.shape
    ldx = x_bf16.stride(0) if M > 1 else K
    if out is None:
        qx = torch.empty((K // 64, M, 32), dtype=torch.uint8, device=x_bf16.device)
        sx = torch.empty(((K // 64 + 1) // 2, M, 2, 2), dtype=torch.uint8, device=x_bf16.device)
        h = torch.empty((M, r), dtype=torch.float32, device=x_bf16.device) if l1_packed is not None else None
    else:
        qx, sx, h = out
    _check(load_library().svdq_quantize_act_mxfp4(_ptr(x_bf16), ldx, _ptr(inv_lambda), float(rho), _ptr(l1_packed),
                                                  M, K, r if l1_packed is not None else 0,
                                                  _ptr(qx), _ptr(sx), _ptr(h), _stream()), "svdq_quantize_act_mxfp4")
    return qx, sx, h


def mx_to_token_major(qx, sx, K):
    """Group-major MXFP4 activations -> (qx [M,K/2], sx [M,K/32]): the layout the format's definition suggests."""
    ng, M, _ = qx.shape
    qx_tm = qx.permute(1, 0, 2).reshape(M, ng * 32).contiguous()
    # sx[s][m][h][j] scales MX block 2 (2s + j) + h  ->  [m][s][j][h]
    sx_tm = sx.permute(1, 0, 3, 2).reshape(M, -1)[:, : K // 32].contiguous()
    return qx_tm, sx_tm


def packed_weight_mxfp4_bytes(N, K):
    return int(load_library().svdq_packed_weight_mxfp4_bytes(N, K))


def pack_weight_mxfp4(qw, sw):
    """qw [N,K/2] u8 packed E2M1 codes, sw [K/32,N] u8 E8M0 bytes (device) -> opaque uint8 tensor for linear_mxfp4."""
    N, K2 = qw.shape
    K = 2 * K2
    out = torch.empty(packed_weight_mxfp4_bytes(N, K), dtype=torch.uint8, device=qw.device)
    _check(load_library().svdq_pack_weight_mxfp4(_ptr(qw), _ptr(sw), N, K, _ptr(out), _stream()), "svdq_pack_weight_mxfp4")
    return out


def linear_mxfp4(qx, sx, w_packed, N, h=None, L2_bf16=None, bias=None, out=None, out_dtype=torch.bfloat16):
    """MXFP4 layer from quantised activations -> y [M,N] bf16 (or f32: the value before the bf16 rounding)."""
    ng, M, _ = qx.shape
    K = 64 * ng
    r = 0 if h is None else h.shape[1]
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=qx.device)
    code = OUT_F32 if out.dtype == torch.float32 else OUT_BF16
    ldy = out.stride(0) if M > 1 else N
    _check(load_library().svdq_linear_mxfp4(_ptr(qx), _ptr(sx), _ptr(w_packed), _ptr(h), _ptr(L2_bf16), _ptr(bias),
                                            M, N, K, r, _ptr(out), ldy, code, _stream()), "svdq_linear_mxfp4")
    return out


def linear_mxfp4_next(qx, sx, w_packed, N, next_inv_lambda, next_rho, h=None, L2_bf16=None, bias=None, gelu=True,
                      next_l1_packed=None, next_r=0, out=None):
    """The MXFP4 layer fused with the NEXT layer's quantise pass (optionally through GELU): returns what
    quantize_act_mxfp4 / quantize_act_gelu(FMT_MXFP4) of this layer's bf16 output would return
    (qx' [N/64,M,32], sx' [N/128,M,2,2], h' [M,next_r] or None), without y ever being stored."""
    ng, M, _ = qx.shape
    K = 64 * ng
    r = 0 if h is None else h.shape[1]
    if out is None:
        nq = torch.empty((N // 64, M, 32), dtype=torch.uint8, device=qx.device)
        ns = torch.empty((N // 128, M, 2, 2), dtype=torch.uint8, device=qx.device)
        nh = torch.empty((M, next_r), dtype=torch.float32, device=qx.device) if next_l1_packed is not None else None
    else:
        nq, ns, nh = out
    _check(load_library().svdq_linear_mxfp4_next(
        _ptr(qx), _ptr(sx), _ptr(w_packed), _ptr(h), _ptr(L2_bf16), _ptr(bias), M, N, K, r, int(bool(gelu)),
        _ptr(next_inv_lambda), float(next_rho), _ptr(next_l1_packed), next_r if next_l1_packed is not None else 0,
        _ptr(nq), _ptr(ns), _ptr(nh), _stream()), "svdq_linear_mxfp4_next")
    return nq, ns, nh


# ---- clipping-ratio search (offline calibration, Sec. III-C) ---------------------------------
def sq_error(y_ref, y, workspace=None, out=None):
    """sum (y_ref - y)^2 over two bf16 [M,N] tensors -> 1-element float64 device tensor."""
    M, N = y.shape
    if workspace is None:
        workspace = torch.empty(load_library().svdq_sq_error_workspace_bytes() // 8, dtype=torch.float64, device=y.device)
    if out is None:
        out = torch.empty(1, dtype=torch.float64, device=y.device)
    _check(load_library().svdq_sq_error(_ptr(y_ref), y_ref.stride(0) if M > 1 else N, _ptr(y), y.stride(0) if M > 1 else N,
                                        M, N, _ptr(workspace), _ptr(out), _stream()), "svdq_sq_error")
    return out


def sq_error_static(y_ref, y, out=None):
    """sq_error through the entry point that allocates nothing and takes no workspace (partial sums in the
    library's static device array)."""
    M, N = y.shape
    if out is None:
        out = torch.empty(1, dtype=torch.float64, device=y.device)
    _check(load_library().svdq_sq_error_static(_ptr(y_ref), y_ref.stride(0) if M > 1 else N, _ptr(y),
                                               y.stride(0) if M > 1 else N, M, N, _ptr(out), _stream()),
           "svdq_sq_error_static")
    return out


def search_clipping_ratios(layer_run, xs, y_refs, bins, nbins, candidates):
    """Timestep-bin clipping-ratio search.  `layer_run(x, rho)` runs the quantised layer (quantise + GEMM kernels)
    and returns y bf16; xs[i], y_refs[i] are the calibration input and full-precision output of step i, bins[i]
    its timestep bin.  Returns (table [nbins] of chosen ratios, err [nbins][len(candidates)] summed errors).
    The sums over a bin's steps and the arg-min over the candidates run in the library, on the device."""
    lib = load_library()
    dev = xs[0].device
    nc = len(candidates)
    ws = torch.empty(lib.svdq_sq_error_workspace_bytes() // 8, dtype=torch.float64, device=dev)
    acc = torch.zeros((nbins, nc), dtype=torch.float64, device=dev)
    idx = torch.empty(nbins, dtype=torch.int32, device=dev)
    for x, yr, b in zip(xs, y_refs, bins):
        M, N = yr.shape
        for ci, rho in enumerate(candidates):
            y = layer_run(x, rho)
            _check(lib.svdq_sq_error_add(_ptr(yr), yr.stride(0) if M > 1 else N, _ptr(y), y.stride(0) if M > 1 else N,
                                         M, N, _ptr(ws), ctypes.c_void_p(acc.data_ptr() + 8 * (b * nc + ci)), _stream()),
                   "svdq_sq_error_add")
    _check(lib.svdq_argmin_rows(_ptr(acc), nbins, nc, _ptr(idx), _stream()), "svdq_argmin_rows")
    table = [float(candidates[i]) for i in idx.cpu().tolist()]
    return table, acc.cpu().numpy()


def debug_scale_chain(a, rho):
    """(s, 1/s) of eq. 8-9 for group magnitudes a (float32 device tensor), from the kernel's device functions."""
    a = a.contiguous()
    s = torch.empty_like(a)
    inv = torch.empty_like(a)
    _check(load_library().svdq_debug_scale_chain(_ptr(a), float(rho), a.numel(), _ptr(s), _ptr(inv), _stream()),
           "svdq_debug_scale_chain")
    return s, inv


_staging = {}        # device -> uint8 tensor shared by every W4A4Linear that keeps its weights in the canonical form


def _staging_buffer(nbytes, device):
    buf = _staging.get(device)
    if buf is None or buf.numel() < nbytes:
        buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
        _staging[device] = buf
    return buf


class W4A4Linear:
    """One quantised linear resident in HBM: weights and low-rank factors, reusable output buffers.

    container "e3m2" (default) runs the int4 layer on the FP6 matrix cores, "nibble" the same layer on 4-bit storage
    and the int8 matrix cores, "mxfp4" the MXFP4 format (qw then holds E2M1 codes and sw [K/32, N] E8M0 bytes).
    resident "w4" (default, container "e3m2" only) keeps the canonical 4-bit weights (qw, sw) and expands them into a
    staging buffer shared by all such layers of the device right before every GEMM (calls on one stream only);
    "packed" keeps the container's own packed form (7 - 8 bits per weight for the int4 containers)."""

    def __init__(self, inv_lambda, L1_bf16, L2_bf16, qw, sw, bias, container="e3m2", resident="w4"):
        assert container in ("e3m2", "nibble", "mxfp4") and resident in ("w4", "packed")
        self.container = container
        self.N, self.K = qw.shape[0], qw.shape[1] * 2
        self.r = 0 if L1_bf16 is None else L1_bf16.shape[1]
        self.inv_lambda = inv_lambda
        self.l1_packed = pack_lowrank_down(L1_bf16, inv_lambda) if self.r else None
        self.L2 = L2_bf16 if self.r else None
        if container == "e3m2" and resident == "w4":
            self.qw, self.sw, self.w_packed = qw, sw, None
        else:
            self.w_packed = {"e3m2": pack_weight_e3m2, "nibble": pack_weight, "mxfp4": pack_weight_mxfp4}[container](qw, sw)
        self.bias = bias
        self._bufs = None

    def weights(self):
        """The packed weights the GEMM takes: resident, or expanded now from the resident 4-bit form."""
        if self.w_packed is not None:
            return self.w_packed
        return pack_weight_e3m2(self.qw, self.sw, out=_staging_buffer(packed_weight_e3m2_bytes(self.N, self.K), self.qw.device))

    def buffers(self, M, device):
        if self._bufs is None or self._bufs[3].shape[0] != M:
            if self.container == "e3m2":
                qx = ActE3M2(torch.empty(act_e3m2_bytes(M, self.K), dtype=torch.uint8, device=device), M, self.K)
                sx = None
            else:
                qx = torch.empty((self.K // 64, M, 32), dtype=torch.uint8, device=device)
                sx = (torch.empty((self.K // 64, M), dtype=torch.float32, device=device) if self.container == "nibble"
                      else torch.empty(((self.K // 64 + 1) // 2, M, 2, 2), dtype=torch.uint8, device=device))
            h = torch.empty((M, self.r), dtype=torch.float32, device=device) if self.r else None
            y = torch.empty((M, self.N), dtype=torch.bfloat16, device=device)
            self._bufs = (qx, sx, h, y)
        return self._bufs

    def quantize(self, x_bf16, rho, gelu=False):
        """Kernel (a) into the layer's buffers; gelu=True applies the feed-forward block's activation on the fly."""
        out = self.buffers(x_bf16.shape[0], x_bf16.device)[:3]
        if gelu:
            fmt = {"e3m2": FMT_INT4_E3M2, "nibble": FMT_INT4, "mxfp4": FMT_MXFP4}[self.container]
            return quantize_act_gelu(fmt, x_bf16, self.inv_lambda, rho, self.l1_packed, self.r, out=out)
        fn = {"e3m2": quantize_act_e3m2, "nibble": quantize_act, "mxfp4": quantize_act_mxfp4}[self.container]
        return fn(x_bf16, self.inv_lambda, rho, self.l1_packed, self.r, out=out)

    def gemm(self, qx, sx, h):
        if self.container == "e3m2":
            y = self.buffers(qx.M, qx.buf.device)[3]
            return linear_w4a4_e3m2(qx, self.weights(), self.N, h, self.L2, self.bias, out=y)
        y = self.buffers(qx.shape[1], qx.device)[3]
        fn = linear_w4a4 if self.container == "nibble" else linear_mxfp4
        return fn(qx, sx, self.w_packed, self.N, h, self.L2, self.bias, out=y)

    def forward(self, x_bf16, rho, gelu=False):
        qx, sx, h = self.quantize(x_bf16, rho, gelu)
        return self.gemm(qx, sx, h)


