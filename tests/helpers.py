"""Test-side helpers: host codecs of the E3M2 activation operand buffer (written from the documented layout,
independent of the library); the device plumbing and the output bar live in workloads/harness.py."""
import numpy as np
import torch

from workloads import synth


from workloads.harness import DeviceLayer, check_y, dev, host_bits, rel_fro  # noqa: F401  (re-exported)


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
