"""ctypes loader for the CPU oracle (oracle/svdq_oracle.cpp).

TEST INFRASTRUCTURE, NOT PRODUCT: only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py import this package.  It holds no arithmetic of
its own: every function marshals numpy arrays into the C entry points declared
in svdq_oracle.h and returns what they wrote.
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


def search_clipping_ratios(layer, xs, y_refs, bins, nbins, candidates, fmt="int4"):
    """For every timestep bin: the candidate ratio with the smallest summed squared reconstruction error of the
    quantised layer over the bin's calibration steps.  `layer` has inv_lambda, L1, L2, qw, sw, bias (numpy);
    xs[i] / y_refs[i] are bf16 bit arrays.  Returns (table, err [nbins][len(candidates)])."""
    err = np.zeros((nbins, len(candidates)), np.float64)
    for x, yr, b in zip(xs, y_refs, bins):
        h = lowrank_down(x, layer.inv_lambda, layer.L1) if layer.r else None
        for ci, rho in enumerate(candidates):
            if fmt == "mxfp4":
                qx, sx = quantize_act_mxfp4(x, layer.inv_lambda, rho)
                y = linear_mxfp4(qx, sx, layer.qw, layer.sw, h, layer.L2 if layer.r else None, layer.bias, want=("ybf16",))
            else:
                qx, sx = quantize_act(x, layer.inv_lambda, rho)
                y = linear(qx, sx, layer.qw, layer.sw, h, layer.L2 if layer.r else None, layer.bias, want=("ybf16",))
            err[b, ci] += sq_error(yr, y["ybf16"])
    table = [float(candidates[int(i)]) for i in err.argmin(axis=1)]
    return table, err


# ---- GPTQ on the residual (Sec. III-B: the residual branch is quantised with GPTQ instead of round-to-nearest) ----
# The paper names the method (Frantar et al.) and gives no formula; this is that algorithm in its plain
# column-sequential form, in binary64, with elementwise operations only (so that a GPU can repeat every bit):
# weights are visited in the order k = 0..K-1; a visited weight is rounded to the int4 grid of its (channel,
# 64-group) scale, and its rounding error is spread over the not yet visited weights of the same channel in
# proportion to the inverse Hessian of the layer-wise objective ||X^ (R - R^)||^2, H = X^T X^ (+ damping), from
# which the visited index is then eliminated.  The published implementation factors H^-1 once (Cholesky) and
# reads the same numbers off the factor; the elimination form below is the definition it is derived from.
def gptq_hessian(x_bf16, inv_lambda):
    """H = X^T X^ in binary64, X^ = x * inv_lambda in binary32 (eq. 5)."""
    from workloads import synth
    xs = (synth.bf16_bits_to_f32(np.asarray(x_bf16)) * np.asarray(inv_lambda, np.float32)[None, :]).astype(np.float64)
    return xs.T @ xs


def gptq_invert(H):
    """In-place Gauss-Jordan inverse without pivoting (H is symmetric positive definite after damping): step p
    divides row p by the pivot, subtracts multiples of it from every other row, and rewrites column p."""
    A = np.array(H, dtype=np.float64)
    K = A.shape[0]
    for p in range(K):
        d = A[p, p]
        col = A[:, p].copy()
        row = A[p] / d                                   # one division per element
        A -= col[:, None] * row[None, :]                 # one product, one subtraction per element
        A[p] = row
        A[:, p] = -col / d
        A[p, p] = 1.0 / d
    return A


def gptq_quantize(R, H, damp=0.01):
    """R [K,N] float32 residual, H [K,K] float64 -> (qw [N,K/2] packed codes, sw [K/64,N] float32 scales).

    Damping: H + damp * mean(diag H) * I; a channel k that no calibration token excites (H[k,k] == 0) gets
    H[k,k] = 1 and R[k,:] = 0.  Scale of a (channel, group): absmax of the group's CURRENT weights when its first
    weight is visited, / 7 in binary32; code = clip(rint(binary32(w) / scale), -8, 7), ties to even."""
    R = np.asarray(R, np.float32)
    K, N = R.shape
    W = R.astype(np.float64)
    Hd = np.array(H, dtype=np.float64)
    dead = np.diag(Hd) == 0
    Hd[dead, dead] = 1.0
    W[dead, :] = 0.0
    acc = 0.0
    for v in np.diag(Hd):                               # summed in index order, so that it can be repeated exactly
        acc += float(v)
    Hd[np.arange(K), np.arange(K)] += damp * (acc / K)
    Hinv = gptq_invert(Hd)
    codes = np.zeros((K, N), np.int8)
    sw = np.zeros((K // 64, N), np.float32)
    s = np.zeros(N, np.float32)
    for i in range(K):
        if i % 64 == 0:
            s = (np.abs(W[i:i + 64]).max(axis=0).astype(np.float32) / np.float32(7.0)).astype(np.float32)
            sw[i // 64] = s
        w = W[i]
        live = s > 0
        safe = np.where(live, s, np.float32(1.0))
        q = np.where(live, np.clip(np.rint(w.astype(np.float32) / safe), -8, 7), 0.0)
        codes[i] = q.astype(np.int8)
        d = Hinv[i, i]
        err = (w - q.astype(np.float64) * s.astype(np.float64)) / d
        if i + 1 < K:
            W[i + 1:] -= Hinv[i, i + 1:, None] * err[None, :]
            Hinv[i + 1:, i + 1:] -= Hinv[i + 1:, i, None] * (Hinv[i, None, i + 1:] / d)
    u = (np.ascontiguousarray(codes.T) & 0xF).astype(np.uint8)
    return (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8), sw


def gptq_objective(R, H, qw, sw):
    """tr((R - R^)^T H (R - R^)) = ||X^ (R - R^)||_F^2 for dequantised R^."""
    from workloads import synth
    K, N = R.shape
    Rq = synth.unpack_int4(qw).T.astype(np.float64) * np.repeat(np.asarray(sw, np.float64), 64, axis=0)
    D = np.asarray(R, np.float64) - Rq
    return float(np.einsum("kn,kj,jn->", D, np.asarray(H, np.float64), D))
