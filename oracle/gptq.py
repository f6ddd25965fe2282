"""Oracle of GPTQ on the residual (Sec. III-B: the residual branch is quantised with GPTQ instead of round-to-nearest).

TEST INFRASTRUCTURE, NOT PRODUCT.  numpy, binary64; shares nothing with the HIP library or the input generators.
"""
import numpy as np


def _bf16_bits_to_f32(b):
    """bf16 bit patterns (uint16) -> float32, exact."""
    return (np.asarray(b).astype(np.uint32) << 16).view(np.float32)


def _unpack_int4(q):
    """[R,K/2] packed two's-complement nibbles (even k in the low nibble) -> [R,K] int8 codes."""
    q = np.asarray(q, np.uint8)
    out = np.empty((q.shape[0], q.shape[1] * 2), np.int16)
    out[:, 0::2] = q & 0xF
    out[:, 1::2] = q >> 4
    return np.where(out >= 8, out - 16, out).astype(np.int8)


# The paper names the method (Frantar et al.) and gives no formula; this is that algorithm in its plain
# column-sequential form, in binary64, with elementwise operations only (so that a GPU can repeat every bit):
# weights are visited in the order k = 0..K-1; a visited weight is rounded to the int4 grid of its (channel,
# 64-group) scale, and its rounding error is spread over the not yet visited weights of the same channel in
# proportion to the inverse Hessian of the layer-wise objective ||X^ (R - R^)||^2, H = X^T X^ (+ damping), from
# which the visited index is then eliminated.  The published implementation factors H^-1 once (Cholesky) and
# reads the same numbers off the factor; the elimination form below is the definition it is derived from.
def gptq_hessian(x_bf16, inv_lambda):
    """H = X^T X^ in binary64, X^ = x * inv_lambda in binary32 (eq. 5)."""
    xs = (_bf16_bits_to_f32(x_bf16) * np.asarray(inv_lambda, np.float32)[None, :]).astype(np.float64)
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
    K, N = R.shape
    Rq = _unpack_int4(qw).T.astype(np.float64) * np.repeat(np.asarray(sw, np.float64), 64, axis=0)
    D = np.asarray(R, np.float64) - Rq
    return float(np.einsum("kn,kj,jn->", D, np.asarray(H, np.float64), D))
