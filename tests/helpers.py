"""Shared plumbing for the GPU parity tests: numpy <-> device tensors, error metrics."""
import numpy as np
import torch

from workloads import synth


def dev(a, dtype=None):
    """numpy array -> cuda tensor; uint16 arrays are reinterpreted as bf16."""
    t = torch.from_numpy(np.ascontiguousarray(a))
    if a.dtype == np.uint16:
        t = t.view(torch.bfloat16)
    return t.cuda()


def host_bits(t):
    """device bf16 tensor -> numpy uint16 bit patterns."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


class DeviceLayer:
    """A synth.Layer uploaded and packed through the C ABI."""

    def __init__(self, L):
        import paper_2605_27003_amd as svdq
        self.L = L
        self.inv_lambda = dev(L.inv_lambda)
        self.L1 = dev(L.L1) if L.r else None
        self.L2 = dev(L.L2) if L.r else None
        self.bias = dev(L.bias)
        self.qw = dev(L.qw)
        self.sw = dev(L.sw)
        self.l1p = svdq.pack_lowrank_down(self.L1, self.inv_lambda) if L.r else None
        self.wp = svdq.pack_weight(self.qw, self.sw)
        self.wp6 = svdq.pack_weight_e3m2(self.qw, self.sw)


E3M2_FIELD = {0: 0, 1: 12, 2: 16, 3: 18, 4: 20, 5: 21, 6: 22, 7: 23, 8: 24}   # |q| -> exponent/mantissa bits


def e3m2_fields(q):
    """int codes in [-8, 8] -> 6-bit E3M2 fields (sign bit 5, 3 exponent bits of bias 3, 2 mantissa bits),
    from the definition of the format: value = (-1)^s 2^(e-3) (1 + m/4), e >= 1 for every nonzero integer."""
    q = np.asarray(q, np.int64)
    a = np.abs(q)
    e = np.where(a > 0, np.floor(np.log2(np.maximum(a, 1))).astype(np.int64), 0)
    m = np.where(a > 0, (a * 4) // (1 << e) - 4, 0)
    assert np.all(np.where(a > 0, (1 << e) * (4 + m), 0) == 4 * a)
    f = np.where(a > 0, ((e + 3) << 2) | m, 0) | np.where(q < 0, 32, 0)
    return f.astype(np.uint8)


def pack_act_e3m2_np(codes, sx):
    """Host-side writer of the activation operand buffer documented in include/svdq.h, from int codes [M, K]
    and binary32 scales [M, K/64].  Independent of the library: used to feed hand-made codes to the GEMM and to
    check the quantise kernel's buffer byte for byte."""
    codes = np.asarray(codes)
    M, K = codes.shape
    ng, Mp = K // 64, (M + 3) // 4 * 4
    f = e3m2_fields(codes).reshape(M, ng, 2, 32).astype(np.uint64)
    bits = np.zeros((M, ng, 2, 3), np.uint64)                      # 192 bits as three 64-bit words, field j at bit 6 j
    for j in range(32):
        w, sh = (6 * j) // 64, (6 * j) % 64
        bits[..., w] |= (f[..., j] << np.uint64(sh)) & np.uint64(0xFFFFFFFFFFFFFFFF)
        if sh > 58:
            bits[..., w + 1] |= f[..., j] >> np.uint64(64 - sh)
    by = bits.view(np.uint8).reshape(M, ng, 2, 24)                 # little-endian bytes of the 24-byte fragment
    buf = np.zeros((ng, Mp * 56), np.uint8)
    p0 = buf[:, : Mp * 32].reshape(ng, Mp, 2, 16)
    p1 = buf[:, Mp * 32: Mp * 48].reshape(ng, 2, Mp, 8)
    p2 = buf[:, Mp * 48:].reshape(ng, Mp, 2, 4)
    p0[:, :M] = by[..., :16].transpose(1, 0, 2, 3)
    p1[:, :, :M] = by[..., 16:].transpose(1, 2, 0, 3)
    s = np.asarray(sx, np.float32)
    hi = synth.to_bf16_bits(s)
    lo = synth.to_bf16_bits((s - synth.bf16_bits_to_f32(hi)).astype(np.float32))
    p2[:, :M] = (hi.astype(np.uint32) | (lo.astype(np.uint32) << 16)).T.copy().view(np.uint8).reshape(ng, M, 1, 4)
    return buf.reshape(-1)


def unpack_act_e3m2_np(buf, M, K):
    """Host-side reader of the same buffer -> (int codes [M, K], scale pieces [M, K/64] uint32).  Fields are
    decoded from the format's definition (negative zero, which the hardware conversion can emit, is 0)."""
    ng, Mp = K // 64, (M + 3) // 4 * 4
    buf = np.asarray(buf, np.uint8).reshape(ng, Mp * 56)
    p0 = buf[:, : Mp * 32].reshape(ng, Mp, 2, 16)[:, :M]
    p1 = buf[:, Mp * 32: Mp * 48].reshape(ng, 2, Mp, 8)[:, :, :M].transpose(0, 2, 1, 3)
    by = np.concatenate([p0, p1], axis=-1)                          # [ng, M, 2, 24]
    bits = np.unpackbits(by, axis=-1, bitorder="little").reshape(ng, M, 2, 32, 6)
    f = (bits * (1 << np.arange(6))).sum(-1)
    e, m, sgn = (f >> 2) & 7, f & 3, f >> 5
    val = np.where(e > 0, (4 + m) * 2.0 ** (e - 5.0), m / 16.0) * np.where(sgn == 1, -1.0, 1.0)
    codes = val.astype(np.int64)
    assert np.array_equal(codes, val), "non-integer field"
    codes = codes.transpose(1, 0, 2, 3).reshape(M, K)
    pair = np.ascontiguousarray(buf[:, Mp * 48:].reshape(ng, Mp, 8)[:, :M]).view(np.uint32).reshape(ng, M, 2)
    assert np.array_equal(pair[..., 0], pair[..., 1]), "scale pieces are stored twice"
    return codes, pair[..., 0].T


def rel_fro(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def check_y(y_gpu_bf16_bits, y_gpu_f32, orc, where=""):
    """The output bar.

    Against the oracle's binary64 y the pre-rounding GPU value must satisfy the
    stated bounds literally: relative Frobenius error <= 2e-3 and max-abs error
    <= 1e-2 * rms(y) (in practice ~1e-5).  The bf16 output must be exactly the
    round-to-nearest-even of that value, must meet the Frobenius bound against
    the oracle's bf16, and may differ from it only by one bf16 step where the
    two pre-rounding values straddle a rounding boundary: one step exceeds
    1e-2*rms for |y| > 2.56 rms, so there the bound is one bf16 ulp.
    """
    y64 = orc["y64"]
    rms = float(np.sqrt(np.mean(y64 ** 2)))
    d32 = y_gpu_f32.astype(np.float64) - y64
    assert np.linalg.norm(d32) / np.linalg.norm(y64) <= 2e-3, where
    assert np.abs(d32).max() <= 1e-2 * rms, where
    # tighter than the stated bar: what the arithmetic should give.  The GEMM adds 2.25*S per group to the
    # fp32 accumulator and removes it every second group, so each FMA rounds at ~2*2.25*2^14 = 7e4 times the
    # unit of one integer accumulator (typical |acc| ~ 80): ~5e-5 relative for K = 5120..13824, plus the
    # 2^-17 of the hi+lo bf16 splits.
    assert np.linalg.norm(d32) / np.linalg.norm(y64) <= 3e-4, (where, "fp32 path far looser than expected")
    want_bits = synth.to_bf16_bits(y_gpu_f32)
    assert np.array_equal(y_gpu_bf16_bits, want_bits), (where, "bf16 output is not RNE of the f32 output")
    yb = synth.bf16_bits_to_f32(y_gpu_bf16_bits).astype(np.float64)
    ob = synth.bf16_bits_to_f32(orc["ybf16"]).astype(np.float64)
    assert np.linalg.norm(yb - ob) / np.linalg.norm(ob) <= 2e-3, where
    ulp = np.maximum(np.abs(ob), 1e-30)
    ulp = 2.0 ** (np.floor(np.log2(ulp)) - 7)
    assert np.all(np.abs(yb - ob) <= np.maximum(1e-2 * rms, ulp * 1.0001)), where
    # how often the two pre-rounding values straddle a bf16 boundary: about E|delta| * E[1/ulp(y)], a few
    # percent for delta ~ 1e-5..1e-4 * rms (small |y| have small ulps).  Reported; a gross value means a bug.
    flips = float(np.mean(yb != ob))
    assert flips <= 0.15, (where, flips)
    stats = {"rel_fro_f32": float(np.linalg.norm(d32) / np.linalg.norm(y64)),
             "max_abs_over_rms": float(np.abs(d32).max() / rms),
             "rel_fro_bf16": float(np.linalg.norm(yb - ob) / np.linalg.norm(ob)), "bf16_flip_frac": flips}
    print(f"[parity] {where}: {stats}", flush=True)
    return stats
