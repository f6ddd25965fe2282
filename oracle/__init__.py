"""ctypes loader for the CPU oracle (oracle/svdq_oracle.cpp).

TEST INFRASTRUCTURE, NOT PRODUCT: only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py import this package.  This module holds no
arithmetic of its own: every function marshals numpy arrays into the C entry
points declared in svdq_oracle.h and returns what they wrote.  The two oracles
written in numpy live in modules of their own and are re-exported at the end:
oracle/gptq.py (GPTQ on the residual, binary64) and oracle/search.py (the
clipping-ratio search loop around the C functions).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "svdq_oracle.cpp")
_LIB = os.path.join(_HERE, "libsvdq_oracle.so")
_lib = None

CXXFLAGS = ["-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math",
            "-shared", "-fPIC", "-pthread"]


def build(force=True):
    """Compile the oracle with g++ (every IEEE binary32 op stays a single op)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    subprocess.check_call(["g++", *CXXFLAGS, "-I", _HERE, _SRC, "-o", _LIB])
    return _LIB


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_LIB)
        L.svdq_oracle_bf16_to_f32.restype = ctypes.c_float
        L.svdq_oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
        L.svdq_oracle_f32_to_bf16.restype = ctypes.c_uint16
        L.svdq_oracle_f32_to_bf16.argtypes = [ctypes.c_float]
        L.svdq_oracle_hw_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def hw_threads():
    return int(lib().svdq_oracle_hw_threads())


def bf16_to_f32(v):
    return float(lib().svdq_oracle_bf16_to_f32(int(v)))


def f32_to_bf16(v):
    return int(lib().svdq_oracle_f32_to_bf16(float(v)))


def alpha_lookup(table, step, step0, nsteps_expert):
    t = np.ascontiguousarray(table, dtype=np.float32)
    f = lib().svdq_oracle_alpha_lookup
    f.restype = ctypes.c_float
    return float(f(_p(t, ctypes.c_float), ctypes.c_int(t.size), ctypes.c_int(step),
                   ctypes.c_int(step0), ctypes.c_int(nsteps_expert)))


def _chk(rc, name):
    if rc != 0:
        raise ValueError(f"{name}: invalid argument (rc={rc})")


def _c(a, dt):
    a = np.ascontiguousarray(a)
    assert a.dtype == dt, (a.dtype, dt)
    return a


def quantize_act(x_bf16, inv_lambda, rho, nthreads=0):
    """x_bf16 [M,K] uint16 (may be a row-strided view) -> (qx [M,K/2] u8, sx [M,K/64] f32)."""
    assert x_bf16.dtype == np.uint16 and x_bf16.ndim == 2 and x_bf16.strides[1] == 2
    M, K = x_bf16.shape
    ldx = x_bf16.strides[0] // 2 if M > 1 else K
    il = _c(inv_lambda, np.float32)
    qx = np.empty((M, K // 2), np.uint8)
    sx = np.empty((M, K // 64), np.float32)
    rc = lib().svdq_oracle_quantize_act(
        _p(x_bf16, ctypes.c_uint16), ctypes.c_int64(ldx), _p(il, ctypes.c_float),
        ctypes.c_float(rho), ctypes.c_int64(M), ctypes.c_int(K),
        _p(qx, ctypes.c_uint8), _p(sx, ctypes.c_float), ctypes.c_int(nthreads))
    _chk(rc, "quantize_act")
    return qx, sx


def lowrank_down(x_bf16, inv_lambda, L1_bf16, nthreads=0):
    """-> h [M,r] float64."""
    assert x_bf16.dtype == np.uint16 and x_bf16.ndim == 2 and x_bf16.strides[1] == 2
    M, K = x_bf16.shape
    ldx = x_bf16.strides[0] // 2 if M > 1 else K
    il = _c(inv_lambda, np.float32)
    L1 = _c(L1_bf16, np.uint16)
    r = L1.shape[1]
    h = np.empty((M, r), np.float64)
    rc = lib().svdq_oracle_lowrank_down(
        _p(x_bf16, ctypes.c_uint16), ctypes.c_int64(ldx), _p(il, ctypes.c_float),
        _p(L1, ctypes.c_uint16), ctypes.c_int64(M), ctypes.c_int(K), ctypes.c_int(r),
        _p(h, ctypes.c_double), ctypes.c_int(nthreads))
    _chk(rc, "lowrank_down")
    return h


def group_acc(qx, qw, nthreads=0):
    """-> acc [M,N,K/64] int32."""
    qx = _c(qx, np.uint8)
    qw = _c(qw, np.uint8)
    M, K2 = qx.shape
    N = qw.shape[0]
    assert qw.shape[1] == K2
    K = 2 * K2
    acc = np.empty((M, N, K // 64), np.int32)
    rc = lib().svdq_oracle_group_acc(
        _p(qx, ctypes.c_uint8), _p(qw, ctypes.c_uint8), ctypes.c_int64(M), ctypes.c_int(N),
        ctypes.c_int(K), _p(acc, ctypes.c_int32), ctypes.c_int(nthreads))
    _chk(rc, "group_acc")
    return acc


def linear(qx, sx, qw, sw, h=None, L2_bf16=None, bias=None, want=("y64", "y32", "ybf16"), nthreads=0):
    """Quantised layer from quantised activations -> dict of requested outputs."""
    qx = _c(qx, np.uint8)
    sx = _c(sx, np.float32)
    qw = _c(qw, np.uint8)
    sw = _c(sw, np.float32)
    M, K2 = qx.shape
    K = 2 * K2
    N = qw.shape[0]
    assert qw.shape == (N, K2) and sx.shape == (M, K // 64) and sw.shape == (K // 64, N)
    r = 0
    if h is not None:
        h = _c(h, np.float64)
        L2_bf16 = _c(L2_bf16, np.uint16)
        r = h.shape[1]
        assert h.shape == (M, r) and L2_bf16.shape == (r, N)
    if bias is not None:
        bias = _c(bias, np.float32)
        assert bias.shape == (N,)
    out = {}
    if "y64" in want:
        out["y64"] = np.empty((M, N), np.float64)
    if "y32" in want:
        out["y32"] = np.empty((M, N), np.float32)
    if "ybf16" in want:
        out["ybf16"] = np.empty((M, N), np.uint16)
    rc = lib().svdq_oracle_linear(
        _p(qx, ctypes.c_uint8), _p(sx, ctypes.c_float), _p(qw, ctypes.c_uint8), _p(sw, ctypes.c_float),
        _p(h, ctypes.c_double), _p(L2_bf16, ctypes.c_uint16), _p(bias, ctypes.c_float),
        ctypes.c_int64(M), ctypes.c_int(N), ctypes.c_int(K), ctypes.c_int(r),
        _p(out.get("y64"), ctypes.c_double), _p(out.get("y32"), ctypes.c_float),
        _p(out.get("ybf16"), ctypes.c_uint16), ctypes.c_int(nthreads))
    _chk(rc, "linear")
    return out


# ---- MXFP4 variant -----------------------------------------------------------
def gelu_tanh_bf16(x_bf16):
    """bf16 bit patterns (any shape) -> bf16 bit patterns of GELU (tanh form) of each value."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    out = np.empty_like(x)
    L = lib()
    L.svdq_oracle_gelu_tanh_bf16.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    L.svdq_oracle_gelu_tanh_bf16.restype = ctypes.c_int
    _chk(L.svdq_oracle_gelu_tanh_bf16(x.ctypes.data_as(ctypes.c_void_p), x.size, out.ctypes.data_as(ctypes.c_void_p)),
         "gelu_tanh_bf16")
    return out


def e2m1_value(code):
    f = lib().svdq_oracle_e2m1_value
    f.restype = ctypes.c_float
    return float(f(ctypes.c_int(int(code))))


def quantize_act_mxfp4(x_bf16, inv_lambda, rho, nthreads=0):
    """x_bf16 [M,K] uint16 -> (qx [M,K/2] u8 packed E2M1 codes, sx [M,K/32] u8 E8M0 scale bytes)."""
    assert x_bf16.dtype == np.uint16 and x_bf16.ndim == 2 and x_bf16.strides[1] == 2
    M, K = x_bf16.shape
    ldx = x_bf16.strides[0] // 2 if M > 1 else K
    il = _c(inv_lambda, np.float32)
    qx = np.empty((M, K // 2), np.uint8)
    sx = np.empty((M, K // 32), np.uint8)
    rc = lib().svdq_oracle_quantize_act_mxfp4(
        _p(x_bf16, ctypes.c_uint16), ctypes.c_int64(ldx), _p(il, ctypes.c_float),
        ctypes.c_float(rho), ctypes.c_int64(M), ctypes.c_int(K),
        _p(qx, ctypes.c_uint8), _p(sx, ctypes.c_uint8), ctypes.c_int(nthreads))
    _chk(rc, "quantize_act_mxfp4")
    return qx, sx


def linear_mxfp4(qx, sx, qw, sw, h=None, L2_bf16=None, bias=None, want=("y64", "y32", "ybf16"), nthreads=0):
    """MXFP4 layer from quantised activations -> dict of requested outputs.  sx [M,K/32] u8, sw [K/32,N] u8."""
    qx = _c(qx, np.uint8)
    sx = _c(sx, np.uint8)
    qw = _c(qw, np.uint8)
    sw = _c(sw, np.uint8)
    M, K2 = qx.shape
    K = 2 * K2
    N = qw.shape[0]
    assert qw.shape == (N, K2) and sx.shape == (M, K // 32) and sw.shape == (K // 32, N)
    r = 0
    if h is not None:
        h = _c(h, np.float64)
        L2_bf16 = _c(L2_bf16, np.uint16)
        r = h.shape[1]
        assert h.shape == (M, r) and L2_bf16.shape == (r, N)
    if bias is not None:
        bias = _c(bias, np.float32)
        assert bias.shape == (N,)
    out = {}
    if "y64" in want:
        out["y64"] = np.empty((M, N), np.float64)
    if "y32" in want:
        out["y32"] = np.empty((M, N), np.float32)
    if "ybf16" in want:
        out["ybf16"] = np.empty((M, N), np.uint16)
    rc = lib().svdq_oracle_linear_mxfp4(
        _p(qx, ctypes.c_uint8), _p(sx, ctypes.c_uint8), _p(qw, ctypes.c_uint8), _p(sw, ctypes.c_uint8),
        _p(h, ctypes.c_double), _p(L2_bf16, ctypes.c_uint16), _p(bias, ctypes.c_float),
        ctypes.c_int64(M), ctypes.c_int(N), ctypes.c_int(K), ctypes.c_int(r),
        _p(out.get("y64"), ctypes.c_double), _p(out.get("y32"), ctypes.c_float),
        _p(out.get("ybf16"), ctypes.c_uint16), ctypes.c_int(nthreads))
    _chk(rc, "linear_mxfp4")
    return out


# ---- clipping-ratio search (Sec. III-C) --------------------------------------------------------
def sq_error(y_ref_bf16, y_bf16):
    a = _c(y_ref_bf16, np.uint16)
    b = _c(y_bf16, np.uint16)
    assert a.shape == b.shape and a.ndim == 2
    f = lib().svdq_oracle_sq_error
    f.restype = ctypes.c_double
    return float(f(_p(a, ctypes.c_uint16), _p(b, ctypes.c_uint16), ctypes.c_int64(a.shape[0]), ctypes.c_int(a.shape[1])))


from .gptq import gptq_hessian, gptq_invert, gptq_objective, gptq_quantize  # noqa: E402,F401
from .search import search_clipping_ratios  # noqa: E402,F401
