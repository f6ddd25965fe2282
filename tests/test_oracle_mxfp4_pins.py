"""Pins for the MXFP4 part of the CPU oracle (the data format of the paper's Table I).

Nothing here comes from the GPU path: closed forms of the format, hand-worked
tie vectors (tests/golden), invariants, brute force with exact rationals.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from workloads import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def bf16(a):
    return synth.to_bf16_bits(np.asarray(a, np.float32))


def f32(b):
    return synth.bf16_bits_to_f32(np.asarray(b, np.uint16))


def nibbles(q):
    out = np.empty((q.shape[0], q.shape[1] * 2), np.uint8)
    out[:, 0::2] = q & 0xF
    out[:, 1::2] = q >> 4
    return out


def e2m1_closed_form(code):
    """sign, 2 exponent bits (bias 1), 1 mantissa bit; exponent field 0 is subnormal."""
    s, e, m = (code >> 3) & 1, (code >> 1) & 3, code & 1
    mag = m * 0.5 if e == 0 else 2.0 ** (e - 1) * (1 + m / 2)
    return -mag if s else mag


def test_e2m1_values_closed_form(oracle):
    for c in range(16):
        v = oracle.e2m1_value(c)
        assert v == e2m1_closed_form(c) and np.signbit(v) == bool(c & 8), c
    assert sorted(abs(oracle.e2m1_value(c)) for c in range(8)) == [0, 0.5, 1, 1.5, 2, 3, 4, 6]


def test_tie_vectors_golden(oracle):
    rows = [l.split() for l in open(os.path.join(GOLD, "mxfp4_tie_vectors.txt")) if l.strip() and l[0] != "#"]
    xv = np.array([float(r[0]) for r in rows], np.float32)
    want = np.array([int(r[1]) for r in rows], np.uint8)
    assert xv.size <= 32
    x = np.zeros((1, 32), np.float32)
    x[0, : xv.size] = xv
    xb = bf16(x)
    # 0.3, 0.7, 1.3 ... are first rounded to bf16, which moves none of them across a rounding boundary
    qx, sx = oracle.quantize_act_mxfp4(xb, np.ones(32, np.float32), 1.0)
    assert sx[0, 0] == 127
    assert np.array_equal(nibbles(qx)[0, : xv.size], want)


@pytest.mark.parametrize("e", [-20, -3, 0, 5])
@pytest.mark.parametrize("top", [4.0, 6.0])
def test_grid_fixed_point(oracle, e, top):
    """Inputs already on the grid (E2M1 value times a power of two, block maximum 4 or 6 times it) come back exactly."""
    rng = np.random.default_rng(3)
    M, K = 5, 128
    codes = rng.integers(0, 16, size=(M, K)).astype(np.uint8)
    codes[:, ::32] = 6 if top == 4.0 else 7                       # every block contains the chosen maximum
    if top == 4.0:
        codes = np.where((codes & 7) == 7, codes - 1, codes).astype(np.uint8)   # nothing above 4
    vals = np.array([e2m1_closed_form(int(c)) for c in codes.ravel()], np.float32).reshape(M, K) * np.float32(2.0 ** e)
    qx, sx = oracle.quantize_act_mxfp4(bf16(vals), np.ones(K, np.float32), 1.0)
    assert np.all(sx == 127 + e)
    got = nibbles(qx)
    # -0 and +0 are both "zero on the grid": compare values, and codes where the value is non-zero
    gv = np.array([e2m1_closed_form(int(c)) for c in got.ravel()], np.float32).reshape(M, K) * np.float32(2.0 ** e)
    assert np.array_equal(gv, vals)
    assert np.array_equal(got[vals != 0], codes[vals != 0])


def test_error_bound_saturation_and_scale_rule(oracle):
    """Per element: error at most half the local E2M1 spacing; beyond 6 X saturation; the shared exponent is
    floor(log2(rho * absmax)) - 2 (checked with exact integer arithmetic on the float's exponent)."""
    rng = np.random.default_rng(5)
    M, K = 16, 256
    x = (rng.standard_normal((M, K)) * np.exp(rng.standard_normal((M, 1)) * 3)).astype(np.float32)
    lam = (rng.random(K) + 0.5).astype(np.float32)
    il = (np.float32(1) / lam).astype(np.float32)
    xb = bf16(x)
    for rho in (1.0, 0.8, 0.6):
        qx, sx = oracle.quantize_act_mxfp4(xb, il, rho)
        xh = (f32(xb) * il[None, :]).astype(np.float32).reshape(M, K // 32, 32)
        a = np.abs(xh).max(axis=2)
        alpha = (np.float32(rho) * a).astype(np.float32)
        expfield = (alpha.view(np.uint32) >> 23) & 0xFF              # floor(log2 alpha) + 127 for normal numbers
        assert np.array_equal(sx.astype(np.int64), expfield.astype(np.int64) - 2)
        X = np.ldexp(1.0, sx.astype(np.int64) - 127)[:, :, None]
        codes = nibbles(qx).reshape(M, K // 32, 32)
        val = np.vectorize(e2m1_closed_form)(codes).astype(np.float64)
        v = xh.astype(np.float64) / X
        mag = np.abs(v)
        spacing = np.where(mag < 2, 0.5, np.where(mag < 4, 1.0, 2.0))
        inside = mag <= 6
        assert np.all(np.abs(val - v)[inside] <= spacing[inside] / 2 + 1e-12)
        assert np.all(np.abs(val)[~inside] == 6)
        assert np.all((np.signbit(val) == np.signbit(xh)))
        if rho == 1.0:
            assert np.all(mag < 8)                                   # the block maximum lands in [4, 8)


def test_rho_lowers_the_shared_exponent_only_across_a_binade(oracle):
    x = np.zeros((1, 32), np.float32)
    x[0, 0] = 4.0
    x[0, 1] = 1.0
    one = np.ones(32, np.float32)
    q1, s1 = oracle.quantize_act_mxfp4(bf16(x), one, 1.0)            # alpha = 4   -> X = 1
    q2, s2 = oracle.quantize_act_mxfp4(bf16(x), one, 0.9)            # alpha = 3.6 -> X = 1/2
    q3, s3 = oracle.quantize_act_mxfp4(bf16(x), one, 0.5)            # alpha = 2   -> X = 1/2
    assert (s1[0, 0], s2[0, 0], s3[0, 0]) == (127, 126, 126)
    assert tuple(nibbles(q1)[0, :2]) == (6, 2)                       # 4 -> 4, 1 -> 1
    assert tuple(nibbles(q2)[0, :2]) == (7, 4)                       # 4 / 0.5 = 8 saturates to 6; 1 / 0.5 = 2


def test_power_of_two_equivariance_and_empty_blocks(oracle):
    rng = np.random.default_rng(7)
    M, K = 6, 128
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[2, 32:64] = 0.0                                                # an all-zero block
    x[4, :] = 0.0                                                    # an all-zero row
    one = np.ones(K, np.float32)
    q0, s0 = oracle.quantize_act_mxfp4(bf16(x), one, 0.9)
    assert s0[2, 1] == 0 and np.all(nibbles(q0)[2, 32:64] == 0)
    assert np.all(s0[4] == 0) and np.all(q0[4] == 0)
    q1, s1 = oracle.quantize_act_mxfp4(bf16(x * np.float32(2.0 ** 7)), one, 0.9)
    live = s0 != 0
    assert np.array_equal(q1, q0) and np.array_equal(s1[live].astype(int), s0[live].astype(int) + 7)
    assert np.all(s1[~live] == 0)
    # a block below the representable scale range is empty
    tiny = np.full((1, 32), 2.0 ** -126, np.float32)
    qt, st_ = oracle.quantize_act_mxfp4(bf16(tiny), np.ones(32, np.float32), 1.0)
    assert st_[0, 0] == 0 and np.all(qt == 0)


def test_linear_is_exact_matmul_of_the_dequantised_operands(oracle):
    """With everything dequantised in binary64 numpy, the layer is a plain matmul: library routine as the pin."""
    rng = np.random.default_rng(11)
    M, K, N, r = 9, 128, 7, 16
    qx = rng.integers(0, 256, size=(M, K // 2)).astype(np.uint8)
    qw = rng.integers(0, 256, size=(N, K // 2)).astype(np.uint8)
    sx = rng.integers(110, 135, size=(M, K // 32)).astype(np.uint8)
    sw = rng.integers(115, 130, size=(K // 32, N)).astype(np.uint8)
    h = rng.standard_normal((M, r))
    L2 = bf16(rng.standard_normal((r, N)))
    bias = rng.standard_normal(N).astype(np.float32)
    out = oracle.linear_mxfp4(qx, sx, qw, sw, h, L2, bias)
    xd = synth.unpack_e2m1(qx).astype(np.float64) * np.repeat(np.ldexp(1.0, sx.astype(int) - 127), 32, axis=1)
    wd = synth.unpack_e2m1(qw).astype(np.float64).T * np.repeat(np.ldexp(1.0, sw.astype(int) - 127), 32, axis=0)
    want = xd @ wd + h @ f32(L2).astype(np.float64) + bias.astype(np.float64)
    assert np.allclose(out["y64"], want, rtol=1e-13, atol=1e-13)
    assert np.array_equal(out["y32"], out["y64"].astype(np.float32))
    assert np.array_equal(out["ybf16"], bf16(out["y32"]))


def test_brute_force_exact_rationals(oracle):
    """Tiny layer, every step in exact rational arithmetic straight from the definitions."""
    rng = np.random.default_rng(13)
    M, K, N = 3, 64, 2
    x = (rng.standard_normal((M, K)) * 3).astype(np.float32)
    xb = bf16(x)
    lam = np.ldexp(1.0, rng.integers(-2, 3, size=K)).astype(np.float32)       # powers of two: x / lambda is exact
    il = (np.float32(1) / lam).astype(np.float32)
    rho = 0.75                                                                 # exact in binary32
    qx, sx = oracle.quantize_act_mxfp4(xb, il, rho)
    grid = [Fraction(0), Fraction(1, 2), Fraction(1), Fraction(3, 2), Fraction(2), Fraction(3), Fraction(4), Fraction(6)]
    codes = nibbles(qx)
    for m in range(M):
        for b in range(K // 32):
            xs = [Fraction(float(f32(xb)[m, k])) / Fraction(float(lam[k])) for k in range(32 * b, 32 * b + 32)]
            alpha = Fraction(rho) * max(abs(v) for v in xs)                    # exact here: few significant bits
            E = 0
            while Fraction(2) ** (E + 1) <= alpha:
                E += 1
            while Fraction(2) ** E > alpha:
                E -= 1
            assert sx[m, b] == E - 2 + 127
            X = Fraction(2) ** (E - 2)
            for i, v in enumerate(xs):
                mag = abs(v) / X
                d = [abs(mag - g) for g in grid]
                best = min(d)
                cands = [c for c in range(8) if d[c] == best]
                c = cands[0] if len(cands) == 1 else [c for c in cands if c % 2 == 0][0]
                if mag > 6:
                    c = 7
                assert codes[m, 32 * b + i] & 7 == c, (m, b, i, float(mag))
                assert (codes[m, 32 * b + i] >> 3) == (1 if v < 0 else 0) or v == 0
    qw = rng.integers(0, 256, size=(N, K // 2)).astype(np.uint8)
    sw = rng.integers(120, 130, size=(K // 32, N)).astype(np.uint8)
    out = oracle.linear_mxfp4(qx, sx, qw, sw)
    wv = nibbles(qw)
    for m in range(M):
        for n in range(N):
            y = Fraction(0)
            for k in range(K):
                vx = Fraction(e2m1_closed_form(int(codes[m, k]))) * Fraction(2) ** (int(sx[m, k // 32]) - 127)
                vw = Fraction(e2m1_closed_form(int(wv[n, k]))) * Fraction(2) ** (int(sw[k // 32, n]) - 127)
                y += vx * vw
            assert abs(Fraction(float(out["y64"][m, n])) - y) <= abs(y) * Fraction(1, 10 ** 12)


def test_generator_weight_format_matches_the_oracle_quantiser(oracle):
    """The input generator's MXFP4 weight quantiser (numpy) and the oracle's activation quantiser (C++) are two
    independent writings of the same conversion rule: on the same numbers they must give the same bytes."""
    rng = np.random.default_rng(17)
    K, N = 256, 12
    R = (rng.standard_normal((K, N)) * np.exp(rng.standard_normal((1, N)) * 2)).astype(np.float32)
    R = f32(bf16(R))                                                           # bf16-exact so both see the same values
    qw, sw = synth.mxfp4_weight(R)
    qx, sx = oracle.quantize_act_mxfp4(bf16(R.T.copy()), np.ones(K, np.float32), 1.0)
    assert np.array_equal(qw, qx) and np.array_equal(sw, sx.T)


def test_end_to_end_error_is_sane(oracle):
    """Report-style sanity: MXFP4 layer vs the dense layer on the tiny workload; low-rank branch helps."""
    w = synth.workload(0, keep_dense=True, fmt="mxfp4")
    L = w.layers["e0/lin"]
    x = w.x["x"]
    dense = f32(x).astype(np.float64) @ L.W.astype(np.float64) + L.bias
    qx, sx = oracle.quantize_act_mxfp4(x, L.inv_lambda, 1.0)
    h = oracle.lowrank_down(x, L.inv_lambda, L.L1)
    y = oracle.linear_mxfp4(qx, sx, L.qw, L.sw, h, L.L2, L.bias)["y64"]
    err = np.linalg.norm(y - dense) / np.linalg.norm(dense)
    assert err < 0.25, err
