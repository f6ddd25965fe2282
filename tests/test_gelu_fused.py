"""GELU fused into the quantise pass: pins of the oracle's activation (CPU) and GPU parity of the fused pass.

The paper does not define the activation of the feed-forward block; it is the model's (GELU, tanh form).  The
oracle evaluates it in binary32 by a fixed operation sequence; it is pinned here against the binary64 definition
through numpy's exp (a different code path), against closed-form properties, and the GPU must reproduce it bit for
bit, after which the fused pass must equal the oracle's quantise pass on the oracle's activated tensor.
"""
import numpy as np
import pytest

import oracle
from workloads import synth

ALL = np.arange(65536, dtype=np.uint16)
with np.errstate(invalid="ignore"):
    XALL = synth.bf16_bits_to_f32(ALL).astype(np.float64)
FINITE = np.isfinite(XALL)


def gelu_ref64(x):
    """binary64 definition in its sigmoid form (1 + tanh cancels catastrophically for negative arguments)."""
    with np.errstate(over="ignore"):
        z = 2.0 * np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)
        return x / (1.0 + np.exp(-z))


def test_oracle_gelu_is_the_correctly_rounded_definition_on_every_bf16_input():
    g = oracle.gelu_tanh_bf16(ALL)
    ref = gelu_ref64(np.where(FINITE, XALL, 0.0))
    want = synth.to_bf16_bits(ref.astype(np.float32))
    diff = (g != want) & FINITE
    # six inputs just below -10 have true values below 1.3e-37 that the oracle flushes to -0
    assert set(np.nonzero(diff)[0].tolist()) <= set(range(0xC120, 0xC126))
    assert np.all(np.abs(ref[diff]) < 1.3e-37) and np.all(g[diff] == 0x8000)
    gv = synth.bf16_bits_to_f32(g).astype(np.float64)
    big = FINITE & (np.abs(ref) > 1e-30)
    ulp = 2.0 ** (np.floor(np.log2(np.abs(ref[big]))) - 7)
    assert np.max(np.abs(gv[big] - ref[big]) / ulp) <= 0.5


def test_oracle_gelu_closed_forms():
    g = oracle.gelu_tanh_bf16(ALL)
    gv = synth.bf16_bits_to_f32(g).astype(np.float64)
    assert g[0x0000] == 0x0000 and g[0x8000] == 0x8000                     # +-0 -> +-0
    pos = FINITE & (XALL >= 6.0)
    assert np.array_equal(g[pos], ALL[pos])                                  # identity once the sigmoid is 1 in bf16
    neg = FINITE & (XALL <= -10.5)
    assert np.all(g[neg] == 0x8000)                                          # -> -0
    assert abs(gv[FINITE].min() + 0.17) < 2e-3 and abs(XALL[FINITE][gv[FINITE].argmin()] + 0.75) < 0.06
    inc = FINITE & (XALL >= -0.7)                                            # non-decreasing right of the minimum
    order = np.argsort(XALL[inc], kind="stable")
    assert np.all(np.diff(gv[inc][order]) >= 0)
    # gelu(x) - gelu(-x) = x, to within the two roundings
    p = FINITE & (XALL > 1e-30) & (XALL < 8)
    xm = synth.to_bf16_bits((-XALL[p]).astype(np.float32))
    d = gv[p] - synth.bf16_bits_to_f32(oracle.gelu_tanh_bf16(xm)).astype(np.float64)
    assert np.all(np.abs(d - XALL[p]) <= 2.0 ** (np.floor(np.log2(XALL[p])) - 7))
    # half of the argument at the origin's tangent: gelu(x) ~ x / 2 for tiny x
    tiny = FINITE & (np.abs(XALL) < 1e-3) & (np.abs(XALL) > 1e-30)
    assert np.all(np.abs(gv[tiny] / XALL[tiny] - 0.5) < 1e-3)


def test_post_gelu_workload_statistic():
    """The down-projection workload is specified as GELU of N(0, 1.5^2): bounded below by -0.17, heavy right tail."""
    z = synth.to_bf16_bits((np.random.default_rng(0).standard_normal(200000) * 1.5).astype(np.float32))
    gv = synth.bf16_bits_to_f32(oracle.gelu_tanh_bf16(z))
    assert gv.min() >= -0.171 and gv.max() > 5.0 and np.mean(gv > 0) > 0.45


# ------------------------------------------------------------------------------------------------ GPU
gpu = pytest.mark.gpu


@pytest.fixture(scope="module")
def svdq():
    import torch

    import paper_2605_27003_amd as m
    m.load_library(build_if_missing=False)
    assert torch.cuda.is_available()
    return m


@gpu
def test_device_gelu_equals_oracle_on_every_finite_bf16(svdq):
    from tests.helpers import dev, host_bits
    got = host_bits(svdq.debug_gelu(dev(ALL)))
    want = oracle.gelu_tanh_bf16(ALL)
    assert np.array_equal(got[FINITE], want[FINITE])


@gpu
@pytest.mark.parametrize("M,K,r", [(333, 1024, 32), (130, 192, 16), (1, 64, 0), (257, 13824, 32)])
def test_fused_pass_equals_oracle_pass_on_activated_tensor(svdq, M, K, r):
    """All three formats: codes and scales bit-exact, h within the bar of the un-fused pass.  The pre-activation
    is N(0, 1.5^2) with a few large channels, so the activated tensor has the post-GELU shape of the workload."""
    import torch

    from tests.helpers import dev, rel_fro, unpack_act_e3m2_np
    z, _ = synth.make_x(100 + M, M, K, outlier_count=3, outlier_scale=8.0, sigma=1.5)
    xg = oracle.gelu_tanh_bf16(z)                                            # what a separate kernel would store
    cm = np.maximum(np.abs(synth.bf16_bits_to_f32(xg)).max(axis=0), 1e-3).astype(np.float32)
    L = synth.make_layer(5, K, 128, r, cm)
    il = dev(L.inv_lambda)
    l1p = svdq.pack_lowrank_down(dev(L.L1), il) if r else None
    rho = 0.8
    oq, os_ = oracle.quantize_act(xg, L.inv_lambda, rho)
    oh = oracle.lowrank_down(xg, L.inv_lambda, L.L1) if r else None
    zt = dev(z)

    def check_h(h):
        if r:
            assert rel_fro(h.cpu().numpy(), oh) <= 3e-5

    qx, sx, h = svdq.quantize_act_gelu(svdq.FMT_INT4, zt, il, rho, l1p, r)
    torch.cuda.synchronize()
    gq, gs = svdq.to_token_major(qx, sx)
    assert np.array_equal(gq.cpu().numpy(), oq) and np.array_equal(gs.cpu().numpy().view(np.uint32), os_.view(np.uint32))
    check_h(h)
    # the fused pass equals the un-fused pass on the activated tensor bit for bit, h included
    q2, s2, h2 = svdq.quantize_act(dev(xg), il, rho, l1p, r)
    assert torch.equal(q2, qx) and torch.equal(s2, sx) and (h is None or torch.equal(h2, h))

    act, sx6, h6 = svdq.quantize_act_gelu(svdq.FMT_INT4_E3M2, zt, il, rho, l1p, r)
    torch.cuda.synchronize()
    codes, _ = unpack_act_e3m2_np(act.buf.cpu().numpy(), M, K)
    assert np.array_equal(codes, synth.unpack_int4(oq)) and torch.equal(sx6, sx)
    check_h(h6)

    qm, sm, hm = svdq.quantize_act_gelu(svdq.FMT_MXFP4, zt, il, rho, l1p, r)
    torch.cuda.synchronize()
    omq, oms = oracle.quantize_act_mxfp4(xg, L.inv_lambda, rho)
    mq, ms = svdq.mx_to_token_major(qm, sm, K)
    assert np.array_equal(mq.cpu().numpy(), omq) and np.array_equal(ms.cpu().numpy(), oms)
    check_h(hm)


@gpu
def test_fused_argument_errors(svdq):
    import torch
    x = torch.zeros((8, 64), dtype=torch.bfloat16, device="cuda")
    il = torch.ones(64, device="cuda")
    with pytest.raises(svdq.SvdqError):
        svdq.quantize_act_gelu(7, x, il, 0.9, out=(torch.zeros(8 * 32, dtype=torch.uint8, device="cuda"),
                                                   torch.zeros(8, device="cuda"), None))
