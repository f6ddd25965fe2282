"""Pins for the CPU oracle: each test checks it against something other than itself.

The paper prints no worked numbers for this path, so the pins are closed forms,
invariants, special cases that reduce to a library routine, hand-worked tie
vectors (tests/golden) and brute force with exact rationals on tiny shapes.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from workloads import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def bf16(a):
    return synth.to_bf16_bits(np.asarray(a, np.float32))


def f32(b):
    return synth.bf16_bits_to_f32(np.asarray(b, np.uint16))


def codes_of(qx):
    return synth.unpack_int4(qx)


# ---------------------------------------------------------------- bf16 casts
def test_bf16_casts_match_torch(oracle):
    rng = np.random.default_rng(1)
    vals = np.concatenate([
        rng.standard_normal(4000).astype(np.float32) * np.float32(3.0),
        np.array([1.00390625, 1.01171875, -1.00390625, 3.0e38, 1e-40, 0.0, -0.0, 65280.0], np.float32),
        (np.float32(1.0) + np.arange(1, 64, dtype=np.float32) * np.float32(2.0 ** -9)),  # exact ties
    ])
    want = torch.from_numpy(vals).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.f32_to_bf16(v) for v in vals], np.uint16)
    assert np.array_equal(got, want)
    back = np.array([oracle.bf16_to_f32(b) for b in want], np.float32)
    assert np.array_equal(back, f32(want))


# ---------------------------------------------------------------- quantiser
def test_tie_vectors_golden(oracle):
    """Sec. III-A eq. 3 with ties to even and clamp to [-8,7]; values in tests/golden/tie_vectors.txt."""
    rows = [l.split() for l in open(os.path.join(GOLD, "tie_vectors.txt")) if l.strip() and l[0] != "#"]
    xv = np.array([float(r[0]) for r in rows], np.float32)
    want = np.array([int(r[1]) for r in rows], np.int8)
    x = np.zeros((1, 64), np.float32)
    x[0, : xv.size] = xv
    qx, sx = oracle.quantize_act(bf16(x), np.ones(64, np.float32), 0.5)
    assert sx[0, 0] == np.float32(1.0)
    assert np.array_equal(codes_of(qx)[0, : xv.size], want)


@pytest.mark.parametrize("e", [-6, -1, 0, 3])
def test_grid_fixed_point(oracle, e):
    """Inputs already on the int4 grid (scale a power of two, a +-7 in every group) come back exactly."""
    rng = np.random.default_rng(50 + e)
    M, K = 7, 256
    q = rng.integers(-7, 8, size=(M, K)).astype(np.int8)
    q[:, ::64] = np.where(rng.random((M, K // 64)) < 0.5, 7, -7)
    s0 = np.float32(2.0 ** e)
    x = q.astype(np.float32) * s0
    qx, sx = oracle.quantize_act(bf16(x), np.ones(K, np.float32), 1.0)
    assert np.all(sx == s0)
    assert np.array_equal(codes_of(qx), q)
    assert np.array_equal(codes_of(qx).astype(np.float32) * sx.repeat(64, axis=1), x)   # zero error


@pytest.mark.parametrize("rho", [1.0, 0.9, 0.6])
def test_half_step_bound_and_clip_count(oracle, rho):
    """|q*s - x^| <= s/2 for unclipped elements; clipped ones sit on the range ends and are counted by brute force."""
    rng = np.random.default_rng(11)
    M, K = 33, 512
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, 17] *= 40
    lam = (0.5 + rng.random(K)).astype(np.float32)
    il = (np.float32(1) / lam).astype(np.float32)
    xb = bf16(x)
    qx, sx = oracle.quantize_act(xb, il, rho)
    q = codes_of(qx).astype(np.float64)
    xh = (f32(xb) * il).astype(np.float64)                 # eq. 5 in binary32, then widened
    s = sx.astype(np.float64).repeat(64, axis=1)
    u = xh / s
    inside = (u > -8.5) & (u < 7.5)
    assert np.all(np.abs(q * s - xh)[inside] <= 0.5 * s[inside] * (1 + 2.0 ** -20))
    assert np.all(q[u >= 7.5 + 1e-4] == 7) and np.all(q[u <= -8.5 - 1e-4] == -8)
    assert q.min() >= -8 and q.max() <= 7
    # the scale is rho * absmax / 7 (eq. 8-9), up to two binary32 roundings
    amax = np.abs(xh).reshape(M, K // 64, 64).max(axis=2)
    assert np.allclose(sx, rho * amax / 7.0, rtol=3e-7, atol=0)
    if rho == 1.0:
        assert inside.all() and q.min() >= -7             # code -8 never appears without clipping
    else:
        assert (~inside).sum() > 0                        # the clipped case is really exercised


def test_zero_and_denormal_groups(oracle):
    x = np.zeros((3, 128), np.float32)
    x[1, 64:] = np.linspace(-1, 1, 64)
    x[2, :64] = 1e-39                                     # bf16-representable denormal range
    qx, sx = oracle.quantize_act(bf16(x), np.ones(128, np.float32), 0.8)
    assert sx[0, 0] == 0 and sx[0, 1] == 0 and sx[1, 0] == 0 and sx[2, 0] == 0 and sx[2, 1] == 0
    assert sx[1, 1] > 0
    c = codes_of(qx)
    assert not c[0].any() and not c[1, :64].any() and not c[2].any() and c[1, 64:].any()


def test_power_of_two_equivariance(oracle):
    rng = np.random.default_rng(3)
    M, K = 9, 192
    x = rng.standard_normal((M, K)).astype(np.float32)
    il = (0.5 + rng.random(K)).astype(np.float32)
    q0, s0 = oracle.quantize_act(bf16(x), il, 0.7)
    q1, s1 = oracle.quantize_act(bf16(x * 8), il, 0.7)
    assert np.array_equal(q0, q1) and np.array_equal(s1, s0 * np.float32(8))
    # scaling channel k of x and lambda_k by the same power of two changes nothing
    e = np.float32(2.0) ** rng.integers(-3, 4, size=K).astype(np.float32)
    q2, s2 = oracle.quantize_act(bf16(x * e), (il / e).astype(np.float32), 0.7)
    assert np.array_equal(q0, q2) and np.array_equal(s0, s2)


def test_in_group_permutation(oracle):
    """Permuting k inside each 64-group (x, lambda, L1 rows, weight rows together) leaves sx, acc and y unchanged."""
    rng = np.random.default_rng(8)
    M, K, N, r = 5, 128, 6, 16
    x = bf16(rng.standard_normal((M, K)))
    il = (0.5 + rng.random(K)).astype(np.float32)
    L1 = bf16(rng.standard_normal((K, r)) * 0.1)
    L2 = bf16(rng.standard_normal((r, N)) * 0.1)
    wq = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    sw = (0.01 + rng.random((K // 64, N))).astype(np.float32)
    perm = np.concatenate([g * 64 + rng.permutation(64) for g in range(K // 64)])

    def pack(c):
        u = (c & 0xF).astype(np.uint8)
        return (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8)

    def run(x, il, L1, wq):
        qx, sx = oracle.quantize_act(x, il, 0.8)
        h = oracle.lowrank_down(x, il, L1)
        acc = oracle.group_acc(qx, pack(wq))
        y = oracle.linear(qx, sx, pack(wq), sw, h, L2, None)["y64"]
        return sx, acc, y

    a = run(x, il, L1, wq)
    b = run(np.ascontiguousarray(x[:, perm]), il[perm], np.ascontiguousarray(L1[perm]), np.ascontiguousarray(wq[:, perm]))
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert np.allclose(a[2], b[2], rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- brute force with exact rationals
def _rhe(fr):
    """round-half-to-even of a Fraction."""
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


def test_brute_force_tiny_exact_rationals(oracle):
    """Sec. III-A eq. 3 and eq. 7 evaluated in exact rational arithmetic on a tiny layer.

    Codes must equal clip(round(x^/s)) computed exactly wherever the exact
    quotient is not within 1e-5 of a rounding boundary (the oracle multiplies by
    RN(1/s), which can differ from the exact quotient by a few ulps); y must
    equal the exact rational value of eq. 7 to binary64 accuracy.
    """
    rng = np.random.default_rng(21)
    M, K, N, r = 4, 128, 3, 16
    xb = bf16(rng.standard_normal((M, K)) * 2)
    il = (0.5 + rng.random(K)).astype(np.float32)
    L1 = bf16(rng.standard_normal((K, r)) * 0.1)
    L2 = bf16(rng.standard_normal((r, N)) * 0.1)
    wq = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    u8 = (wq & 0xF).astype(np.uint8)
    qw = (u8[:, 0::2] | (u8[:, 1::2] << 4)).astype(np.uint8)
    sw = (0.01 + rng.random((K // 64, N))).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    rho = 0.8

    qx, sx = oracle.quantize_act(xb, il, rho)
    h = oracle.lowrank_down(xb, il, L1)
    out = oracle.linear(qx, sx, qw, sw, h, L2, bias)
    q = codes_of(qx)

    xh32 = f32(xb) * il                                    # one binary32 multiply (eq. 5)
    checked = 0
    for m in range(M):
        for g in range(K // 64):
            grp = [Fraction(float(v)) for v in xh32[m, g * 64:(g + 1) * 64]]
            a = max(abs(v) for v in grp)
            s_exact = Fraction(float(np.float32(rho))) * a / 7
            s = Fraction(float(sx[m, g]))
            assert abs(s - s_exact) <= s_exact * Fraction(1, 2 ** 22)
            for i, v in enumerate(grp):
                uq = v / s
                near = min(abs(uq - (k + Fraction(1, 2))) for k in range(-10, 10))
                if near < Fraction(1, 100000):
                    continue
                want = max(-8, min(7, _rhe(uq)))
                assert q[m, g * 64 + i] == want
                checked += 1
    assert checked > M * K * 0.99

    L1f = [[Fraction(float(v)) for v in row] for row in f32(L1)]
    L2f = [[Fraction(float(v)) for v in row] for row in f32(L2)]
    for m in range(M):
        hx = [sum(Fraction(float(xh32[m, k])) * L1f[k][j] for k in range(K)) for j in range(r)]
        for j in range(r):
            assert abs(float(hx[j]) - h[m, j]) <= 1e-12 * (1 + abs(float(hx[j])))
        for n in range(N):
            y = Fraction(float(bias[n]))
            for g in range(K // 64):
                acc = sum(int(q[m, k]) * int(wq[n, k]) for k in range(g * 64, (g + 1) * 64))
                y += acc * Fraction(float(sx[m, g])) * Fraction(float(sw[g, n]))
            y += sum(hx[j] * L2f[j][n] for j in range(r))
            yf = float(y)
            assert abs(out["y64"][m, n] - yf) <= 1e-12 * (1 + abs(yf))
            assert out["y32"][m, n] == np.float32(out["y64"][m, n])
            want_b = torch.tensor([out["y32"][m, n]]).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)[0]
            assert out["ybf16"][m, n] == want_b


# ---------------------------------------------------------------- special cases that are library routines
def test_integer_gemm_special_case(oracle):
    """All scales 1, no low-rank, no bias: the layer is a plain integer matrix product."""
    rng = np.random.default_rng(4)
    M, K, N = 19, 320, 23
    a = rng.integers(-8, 8, size=(M, K)).astype(np.int8)
    w = rng.integers(-8, 8, size=(N, K)).astype(np.int8)

    def pack(c):
        u = (c & 0xF).astype(np.uint8)
        return (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8)

    ng = K // 64
    out = oracle.linear(pack(a), np.ones((M, ng), np.float32), pack(w), np.ones((ng, N), np.float32))
    want = a.astype(np.int64) @ w.astype(np.int64).T
    assert np.array_equal(out["y64"], want.astype(np.float64))
    assert np.array_equal(out["y32"], want.astype(np.float32))
    acc = oracle.group_acc(pack(a), pack(w))
    want_g = np.einsum("mgk,ngk->mng", a.reshape(M, ng, 64).astype(np.int64), w.reshape(N, ng, 64).astype(np.int64))
    assert np.array_equal(acc, want_g.astype(np.int32))
    # extreme codes: every product 64, every group 4096
    e = np.full((2, 64), -8, np.int8)
    assert oracle.group_acc(pack(e), pack(e))[0, 0, 0] == 4096


def test_lowrank_down_is_a_matmul(oracle):
    rng = np.random.default_rng(6)
    M, K, r = 11, 192, 32
    xb = bf16(rng.standard_normal((M, K)))
    il = (0.5 + rng.random(K)).astype(np.float32)
    L1 = bf16(rng.standard_normal((K, r)))
    h = oracle.lowrank_down(xb, il, L1)
    want = (f32(xb) * il).astype(np.float64) @ f32(L1).astype(np.float64)
    assert np.allclose(h, want, rtol=1e-13, atol=1e-13)


def test_full_rank_reconstruction(oracle):
    """r = full rank and residual 0 => the layer returns x W + b (eq. 5-7 with R = 0).

    lambda is a power of two per channel so that D W and x D^-1 are exact; this
    fails if W were scaled by 1/lambda instead of lambda.
    """
    rng = np.random.default_rng(9)
    M, K, N = 13, 64, 64
    xb = bf16(rng.standard_normal((M, K)))
    W = f32(bf16(rng.standard_normal((K, N)) * 0.05))
    lam = (np.float32(2.0) ** rng.integers(-2, 3, size=K)).astype(np.float32)
    What = lam[:, None] * W                                # D W, still bf16-representable
    L1 = bf16(What)
    assert np.array_equal(f32(L1), What)
    L2 = bf16(np.eye(N, dtype=np.float32))
    bias = rng.standard_normal(N).astype(np.float32)
    il = (np.float32(1) / lam).astype(np.float32)
    qx, sx = oracle.quantize_act(xb, il, 0.9)
    h = oracle.lowrank_down(xb, il, L1)
    qw = np.zeros((N, K // 2), np.uint8)                    # R = 0
    sw = np.ones((1, N), np.float32)
    y = oracle.linear(qx, sx, qw, sw, h, L2, bias)["y64"]
    want = f32(xb).astype(np.float64) @ W.astype(np.float64) + bias.astype(np.float64)
    assert np.allclose(y, want, rtol=1e-13, atol=1e-13)
    # r = 0: main branch + bias only
    y0 = oracle.linear(qx, sx, qw, sw, None, None, bias)["y64"]
    assert np.allclose(y0, np.broadcast_to(bias.astype(np.float64), (M, N)))


def test_alpha_lookup_brute_force(oracle):
    table = [0.6, 0.7, 0.8, 0.9, 1.0, 0.8, 0.9, 0.7]
    for nbins in (1, 4, 8):
        for step0, n in ((0, 20), (20, 20), (0, 40), (3, 7)):
            for step in range(step0, step0 + n):
                want = table[int(Fraction(step - step0, n) * nbins)]
                assert oracle.alpha_lookup(table[:nbins], step, step0, n) == np.float32(want)
            assert np.isnan(oracle.alpha_lookup(table[:nbins], step0 - 1, step0, n))
            assert np.isnan(oracle.alpha_lookup(table[:nbins], step0 + n, step0, n))


# ---------------------------------------------------------------- end to end on the tiny workload
def test_end_to_end_against_dense(oracle):
    """The quantised layer approximates x W + b, and the low-rank branch helps (ordering of Table I)."""
    w = synth.workload(0, keep_dense=True)
    L = w.layers["e0/lin"]
    x = w.x["x"]
    dense = f32(x).astype(np.float64) @ L.W.astype(np.float64) + L.bias
    qx, sx = oracle.quantize_act(x, L.inv_lambda, 0.9)
    h = oracle.lowrank_down(x, L.inv_lambda, L.L1)
    y = oracle.linear(qx, sx, L.qw, L.sw, h, L.L2, L.bias)["y64"]
    err = np.linalg.norm(y - dense) / np.linalg.norm(dense)
    # same weights, no low-rank branch: residual = the whole smoothed weight
    qw0, sw0 = synth.rtn_int4_weight((L.lam[:, None] * L.W).astype(np.float32))
    y0 = oracle.linear(qx, sx, qw0, sw0, None, None, L.bias)["y64"]
    err0 = np.linalg.norm(y0 - dense) / np.linalg.norm(dense)
    assert err < 0.12 and err < err0
