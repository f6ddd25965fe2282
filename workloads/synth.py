"""Seeded synthetic inputs for the W4A4 SVDQuant-style linear layer.

This module only MAKES INPUTS.  It serves both the CPU oracle and the GPU
library (the same arrays are handed to each) and holds none of the run-time
path's arithmetic: no activation quantiser, no integer GEMM, no dequantisation,
no low-rank product.  What it does hold is the OFFLINE side the paper treats
as calibration output (Sec. III-B): the smoothing vector of eq. 5, the low-rank
split of eq. 6 and a round-to-nearest int4 residual (the format GPTQ would also
emit), because the layer needs such tensors as inputs.

Shapes follow Wan2.2-A14B (hidden 5120, FFN 13824, 32760 tokens at 480p and
75600 at 720p).  Values are synthetic stand-ins for the paper's calibration and
evaluation data, which are not available: Gaussian bulk plus sparse
channel-wise outliers (Sec. I), post-GELU inputs for the FFN down-projection,
and clipping-ratio tables shaped like Fig. 3 (mostly 0.8, some 0.9).
All randomness comes from numpy's counter-based Philox generator.
"""
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np
import torch

GROUP = 64
RATIOS = (0.6, 0.7, 0.8, 0.9, 1.0)       # candidate set R of eq. 10


def _rng(seed, stream):
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 array -> bf16 bit patterns (uint16), round-to-nearest-even (torch's cast)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


# --------------------------------------------------------------------------
# activations
# --------------------------------------------------------------------------
def make_x(seed: int, M: int, K: int, kind: str = "normal",
           outlier_frac: float = 0.0, outlier_count: int = 0, outlier_scale: float = 1.0,
           heavy_count: int = 0, heavy_scale: float = 1.0, sigma: float = 1.0,
           chunk_rows: int = 4096, value_seed: Optional[int] = None):
    """Activation matrix as bf16 bits [M,K] plus the per-channel max |x| (float32).

    kind "normal": N(0, sigma^2); kind "gelu": GELU(z), z ~ N(0, sigma^2).
    `outlier_count` (or round(outlier_frac*K)) channels are scaled by
    outlier_scale, a further `heavy_count` channels by heavy_scale; channels are
    drawn without replacement from the same generator.  `value_seed` (default:
    `seed`) keys the value streams only: the outlier channels stay those of `seed`.
    """
    g_ch = _rng(seed, 1)
    n_out = outlier_count if outlier_count else int(round(outlier_frac * K))
    chans = g_ch.permutation(K)
    mult = np.ones(K, np.float32)
    mult[chans[:n_out]] = outlier_scale
    mult[chans[n_out:n_out + heavy_count]] = heavy_scale
    x = np.empty((M, K), np.uint16)
    bounds = list(range(0, M, chunk_rows))

    def fill(ci):
        # every chunk has its own counter-based stream, so the result does not depend on the thread count
        m0 = bounds[ci]
        m1 = min(M, m0 + chunk_rows)
        g = np.random.Generator(np.random.Philox(key=[int(seed if value_seed is None else value_seed), 2 + (ci << 8)]))
        z = g.standard_normal((m1 - m0, K), dtype=np.float32)
        if sigma != 1.0:
            z *= np.float32(sigma)
        if kind == "gelu":
            z = torch.nn.functional.gelu(torch.from_numpy(z)).numpy()
        elif kind != "normal":
            raise ValueError(kind)
        z *= mult
        xb = to_bf16_bits(z)
        x[m0:m1] = xb
        return np.abs(bf16_bits_to_f32(xb)).max(axis=0)

    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
        colmax = np.zeros(K, np.float32)
        for cm in ex.map(fill, range(len(bounds))):
            np.maximum(colmax, cm, out=colmax)
    return x, colmax


# --------------------------------------------------------------------------
# offline side: smoothing vector, low-rank split, int4 residual
# --------------------------------------------------------------------------
def _lowrank(What: np.ndarray, r: int, seed: int):
    """Rank-r factors of What [K,N]: exact SVD when small, randomised range finder otherwise."""
    K, N = What.shape
    if min(K, N) <= 1024:
        U, S, Vt = np.linalg.svd(What.astype(np.float64), full_matrices=False)
    else:
        g = _rng(seed, 7)
        Y = What @ g.standard_normal((N, r + 8), dtype=np.float32)
        for _ in range(2):
            Q, _ = np.linalg.qr(Y)
            Y = What @ (What.T @ Q)
        Q, _ = np.linalg.qr(Y)
        Ub, S, Vt = np.linalg.svd((Q.T @ What).astype(np.float64), full_matrices=False)
        U = Q.astype(np.float64) @ Ub
    rs = np.sqrt(S[:r])
    return (U[:, :r] * rs).astype(np.float32), (rs[:, None] * Vt[:r]).astype(np.float32)


def rtn_int4_weight(R: np.ndarray):
    """R [K,N] float32 -> (qw [N,K/2] packed codes, sw [K/64,N] float32 scales).

    Per output channel, per 64-group along K: scale = absmax/7, code =
    clip(rint(R/scale), -8, 7) with ties to even; low nibble holds the even k.
    """
    K, N = R.shape
    ng = K // GROUP
    Rg = R.reshape(ng, GROUP, N)
    sw = (np.abs(Rg).max(axis=1) / np.float32(7.0)).astype(np.float32)        # [ng,N]
    safe = np.where(sw > 0, sw, np.float32(1.0))
    q = np.clip(np.rint(Rg / safe[:, None, :]), -8, 7).astype(np.int8)         # [ng,64,N]
    q = np.where(sw[:, None, :] > 0, q, 0).astype(np.int8)
    qT = np.ascontiguousarray(q.reshape(K, N).T)                                # [N,K]
    u = (qT & 0xF).astype(np.uint8)
    qw = (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8)
    return qw, sw


MX_BLOCK = 32
E2M1_VALUES = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], np.float32)


def mxfp4_weight(R: np.ndarray):
    """R [K,N] float32 -> (qw [N,K/2] packed E2M1 codes, sw [K/32,N] uint8 E8M0 scale bytes).

    Microscaling FP4 per output channel, per 32-block along K: shared exponent
    floor(log2(absmax)) - 2, element = nearest E2M1 value of R / 2^shared (ties
    to the even code, saturating at 6); an all-zero block gets byte 0, codes 0.
    """
    K, N = R.shape
    nb = K // MX_BLOCK
    Rb = R.reshape(nb, MX_BLOCK, N).astype(np.float32)
    amax = np.abs(Rb).max(axis=1)                                              # [nb,N]
    live = amax >= np.float32(2.0 ** -124)
    _, E = np.frexp(np.where(live, amax, np.float32(1.0)))                     # amax = f * 2^E, f in [0.5,1)
    shared = (E - 1) - 2
    X = np.ldexp(np.float32(1.0), shared).astype(np.float32)
    v = np.abs(Rb) / X[:, None, :]
    code = ((v > 0.25).astype(np.uint8) + (v >= 0.75) + (v > 1.25) + (v >= 1.75) + (v > 2.5) + (v >= 3.5)
            + (v > 5.0)).astype(np.uint8)
    code |= (np.signbit(Rb).astype(np.uint8) << 3)
    code = np.where(live[:, None, :], code, 0).astype(np.uint8)
    sw = np.where(live, shared + 127, 0).astype(np.uint8)
    cT = np.ascontiguousarray(code.reshape(K, N).T)                             # [N,K]
    qw = (cT[:, 0::2] | (cT[:, 1::2] << 4)).astype(np.uint8)
    return qw, sw


def unpack_e2m1(q: np.ndarray) -> np.ndarray:
    """[R,K/2] packed E2M1 codes -> [R,K] float32 values."""
    out = np.empty((q.shape[0], q.shape[1] * 2), np.uint8)
    out[:, 0::2] = q & 0xF
    out[:, 1::2] = q >> 4
    v = E2M1_VALUES[out & 7]
    return np.where(out & 8, -v, v).astype(np.float32)


def pack_int4(c: np.ndarray) -> np.ndarray:
    """[R,K] signed codes in [-8,7] -> [R,K/2] packed (even k in the low nibble)."""
    u = (np.asarray(c).astype(np.int16) & 0xF).astype(np.uint8)
    return (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8)


def unpack_int4(q: np.ndarray) -> np.ndarray:
    """[R,K/2] packed -> [R,K] int8 signed codes."""
    lo = (q & 0xF).astype(np.int8)
    hi = (q >> 4).astype(np.int8)
    lo = np.where(lo >= 8, lo - 16, lo).astype(np.int8)
    hi = np.where(hi >= 8, hi - 16, hi).astype(np.int8)
    out = np.empty((q.shape[0], q.shape[1] * 2), np.int8)
    out[:, 0::2] = lo
    out[:, 1::2] = hi
    return out


@dataclass
class Layer:
    """Static tensors of one quantised linear (what calibration would hand over)."""
    K: int
    N: int
    r: int
    lam: np.ndarray            # [K] f32, diagonal of D in eq. 5
    inv_lambda: np.ndarray     # [K] f32, RN(1/lam)
    L1: np.ndarray             # [K,r] bf16 bits
    L2: np.ndarray             # [r,N] bf16 bits
    qw: np.ndarray             # [N,K/2] packed 4-bit codes of the residual (int4, or E2M1 for fmt "mxfp4")
    sw: np.ndarray             # int4: [K/64,N] f32 scales; mxfp4: [K/32,N] uint8 E8M0 bytes
    bias: np.ndarray           # [N] f32
    W: Optional[np.ndarray] = None   # dense [K,N] f32, only kept on request
    fmt: str = "int4"
    qw_mx: Optional[np.ndarray] = None   # fmt "both": the same residual also as E2M1 codes ...
    sw_mx: Optional[np.ndarray] = None   # ... and E8M0 bytes [K/32,N] (qw, sw then hold the int4 form)


def make_layer(seed: int, K: int, N: int, r: int, x_colmax: np.ndarray,
               w_outlier_cols: int = 0, w_outlier_scale: float = 1.0,
               keep_dense: bool = False, fmt: str = "int4") -> Layer:
    g = _rng(seed, 3)
    W = g.standard_normal((K, N), dtype=np.float32) * np.float32(0.02)
    if w_outlier_cols:
        cols = _rng(seed, 4).permutation(N)[:w_outlier_cols]
        W[:, cols] *= np.float32(w_outlier_scale)
    wmax = np.abs(W).max(axis=1)
    lam = np.sqrt(np.maximum(x_colmax, np.float32(1e-6)) / wmax).astype(np.float32)
    inv_lambda = (np.float32(1.0) / lam).astype(np.float32)
    What = lam[:, None] * W                                   # D W of eq. 5
    if r > 0:
        L1f, L2f = _lowrank(What, r, seed)
        L1 = to_bf16_bits(L1f)
        L2 = to_bf16_bits(L2f)
        R = What - bf16_bits_to_f32(L1) @ bf16_bits_to_f32(L2)   # eq. 6 with the stored factors
    else:
        L1 = np.zeros((K, 0), np.uint16)
        L2 = np.zeros((0, N), np.uint16)
        R = What
    R = R.astype(np.float32)
    qw, sw = (mxfp4_weight if fmt == "mxfp4" else rtn_int4_weight)(R)
    qw_mx, sw_mx = mxfp4_weight(R) if fmt == "both" else (None, None)
    bias = (_rng(seed, 5).standard_normal(N, dtype=np.float32) * np.float32(0.01)).astype(np.float32)
    return Layer(K, N, r, lam, inv_lambda, L1, L2, qw, sw, bias, W if keep_dense else None, fmt, qw_mx, sw_mx)


# --------------------------------------------------------------------------
# the five workloads
# --------------------------------------------------------------------------
# inputs of the DiT block workload: name -> (seed, K, make_x arguments)
BLOCK_INPUTS = {
    "x_qkv": (50, 5120, dict(outlier_frac=0.005, outlier_scale=50.0)),
    "x_o": (51, 5120, dict(outlier_frac=0.005, outlier_scale=50.0)),
    "x_up": (52, 5120, dict(outlier_frac=0.005, outlier_scale=50.0, heavy_count=8, heavy_scale=100.0)),
    "x_down": (53, 13824, dict(kind="gelu", sigma=1.5)),
}


def block_input(name: str, M: int, step: Optional[int] = None):
    """Input `name` of the DiT block workload: (bf16 bits [M,K], per-channel max).  step=None is the base input the
    layers were calibrated on; a denoising step number draws fresh values of the same distribution (seed + 1000 *
    (step + 1)) with the SAME outlier channels (the channel pattern belongs to the layer, not to the step)."""
    seed, K, kw = BLOCK_INPUTS[name]
    if step is None:
        return make_x(seed, M, K, **kw)
    return make_x(seed, M, K, value_seed=seed + 1000 * (step + 1), **kw)


@dataclass
class Workload:
    name: str
    M: int
    x: Dict[str, np.ndarray]                 # input name -> bf16 bits [M,K]
    layers: Dict[str, Layer]                 # "<expert>/<linear>" -> Layer
    inputs_of: Dict[str, str]                # linear name -> input name
    tables: Dict[str, List[float]]           # expert -> clipping ratio per timestep bin
    nsteps: int = 1                          # denoising steps in the schedule
    switch_step: int = 0                     # first step of the second expert
    experts: List[str] = field(default_factory=lambda: ["e0"])


def _table(seed, nbins, probs=None):
    g = _rng(seed, 6)
    return [float(v) for v in g.choice(RATIOS, size=nbins, p=probs)]


def workload(idx: int, M: Optional[int] = None, keep_dense: bool = False, fmt: str = "int4") -> Workload:
    """Workload `idx` (0-based; the five configurations of the benchmark definition).

    `M` overrides the token count (tests use it for row-reduced variants that
    keep K, N, r and the value distributions).  fmt "int4" / "mxfp4" selects the
    residual's 4-bit format; "both" quantises the same residual both ways (one
    synthesis serves every execution a benchmark times).
    """
    if idx == 0:
        M = M or 256
        x, cm = make_x(0, M, 512, outlier_count=4, outlier_scale=40.0)
        L = make_layer(0, 512, 512, 16, cm, w_outlier_cols=4, w_outlier_scale=10.0, keep_dense=keep_dense, fmt=fmt)
        return Workload("c1_tiny", M, {"x": x}, {"e0/lin": L}, {"lin": "x"}, {"e0": [0.9]})
    if idx == 1:
        M = M or 32760
        x, cm = make_x(2, M, 5120, outlier_frac=0.005, outlier_scale=50.0)
        L = make_layer(2, 5120, 5120, 32, cm, keep_dense=keep_dense, fmt=fmt)
        return Workload("c2_attn_o", M, {"x": x}, {"e0/lin": L}, {"lin": "x"}, {"e0": _table(2, 4)})
    if idx == 2:
        M = M or 32760
        x, cm = make_x(3, M, 5120, outlier_frac=0.005, outlier_scale=50.0, heavy_count=8, heavy_scale=100.0)
        L = make_layer(3, 5120, 13824, 32, cm, keep_dense=keep_dense, fmt=fmt)
        return Workload("c3_ffn_up", M, {"x": x}, {"e0/lin": L}, {"lin": "x"}, {"e0": [0.9, 0.8, 0.8, 0.9]})
    if idx == 3:
        M = M or 32760
        x, cm = make_x(4, M, 13824, kind="gelu", sigma=1.5)
        L = make_layer(4, 13824, 5120, 32, cm, keep_dense=keep_dense, fmt=fmt)
        return Workload("c4_ffn_down", M, {"x": x}, {"e0/lin": L}, {"lin": "x"}, {"e0": [0.8, 0.8, 0.7, 0.8]})
    if idx == 4:
        M = M or 75600
        xs, cms = {}, {}
        for name in BLOCK_INPUTS:
            xs[name], cms[name] = block_input(name, M)
        shapes = {"q": ("x_qkv", 5120, 5120), "k": ("x_qkv", 5120, 5120), "v": ("x_qkv", 5120, 5120),
                  "o": ("x_o", 5120, 5120), "ffn_up": ("x_up", 5120, 13824), "ffn_down": ("x_down", 13824, 5120)}
        layers, tables, jobs = {}, {}, []
        for e, ename in enumerate(("high_noise", "low_noise")):
            for j, (lin, (inp, K, N)) in enumerate(shapes.items()):
                jobs.append((f"{ename}/{lin}", 500 + 10 * e + j, K, N, cms[inp]))
            tables[ename] = _table(540 + e, 8, probs=[0.05, 0.1, 0.55, 0.25, 0.05])
        with ThreadPoolExecutor(max_workers=4) as ex:
            made = ex.map(lambda j: make_layer(j[1], j[2], j[3], 32, j[4], keep_dense=keep_dense, fmt=fmt), jobs)
            for job, L in zip(jobs, made):
                layers[job[0]] = L
        return Workload("c5_block_720p", M, xs, layers, {k: v[0] for k, v in shapes.items()}, tables,
                        nsteps=40, switch_step=20, experts=["high_noise", "low_noise"])
    raise ValueError(f"no workload {idx}")


def sample_rows(M: int, n_random: int, seed: int, edge: int = 64) -> np.ndarray:
    """Row sample for full-size parity: the first and last `edge` rows plus random rows."""
    edge = min(edge, M // 2)
    fixed = np.concatenate([np.arange(edge), np.arange(M - edge, M)])
    rest = np.setdiff1d(np.arange(M), fixed)
    n_random = min(n_random, rest.size)
    rnd = _rng(seed, 9).choice(rest, size=n_random, replace=False) if n_random else np.empty(0, np.int64)
    return np.sort(np.concatenate([fixed, rnd])).astype(np.int64)
