"""GPTQ on the residual weights (Sec. III-B): pins of the oracle (CPU) and GPU parity.

The paper names the algorithm and prints no formula.  The oracle is its column-sequential definition in binary64
with elementwise updates; pins: with an identity Hessian nothing propagates and the result is round-to-nearest
(the int4 weight format of the layer); a two-weight case against the closed form worked out here; the inverse
against numpy's; the layer-wise objective never above round-to-nearest's on correlated activations; the
error-feedback property that distinguishes it from rounding.  GPU: bit-exact codes and scales.
"""
import numpy as np
import pytest

import oracle
from workloads import synth


def correlated_hessian(seed, M, K):
    rng = np.random.default_rng(seed)
    base = rng.standard_normal((M, 8))
    X = (base @ rng.standard_normal((8, K)) + 0.3 * rng.standard_normal((M, K))).astype(np.float32)
    xb = synth.to_bf16_bits(X)
    il = np.ones(K, np.float32)
    return xb, il, oracle.gptq_hessian(xb, il)


def test_identity_hessian_is_round_to_nearest():
    rng = np.random.default_rng(1)
    R = (rng.standard_normal((256, 96)) * 0.02).astype(np.float32)
    R[64:128, 5] = 0.0                                              # an empty group
    qw, sw = oracle.gptq_quantize(R, np.eye(256), damp=0.0)
    rq, rs = synth.rtn_int4_weight(R)
    assert np.array_equal(qw, rq) and np.array_equal(sw.view(np.uint32), rs.view(np.uint32))


def test_inverse_matches_numpy():
    _, _, H = correlated_hessian(2, 500, 128)
    H += 0.01 * np.mean(np.diag(H)) * np.eye(128)
    A = oracle.gptq_invert(H)
    assert np.abs(A @ H - np.eye(128)).max() < 1e-9 and np.abs(A - np.linalg.inv(H)).max() <= 1e-9 * np.abs(A).max()


def test_two_weights_closed_form():
    """K = 64 with only weights 0 and 1 nonzero and everything else decoupled: the second weight is rounded after
    receiving -e0 * Hinv[0,1] / Hinv[0,0], where e0 is the first weight's rounding error."""
    K = 64
    H = np.eye(K)
    H[0, 1] = H[1, 0] = 0.6
    R = np.zeros((K, 1), np.float32)
    R[0, 0], R[1, 0] = 0.70, 0.33                                    # scale = 0.7 / 7 = 0.1
    qw, sw = oracle.gptq_quantize(R, H, damp=0.0)
    c = synth.unpack_int4(qw)[0]
    s = float(sw[0, 0])
    assert c[0] == 7 and abs(s - np.float32(0.7) / np.float32(7)) == 0
    Hinv = np.linalg.inv(H[:2, :2])
    e0 = float(np.float32(0.70)) - 7 * s
    w1 = float(np.float32(0.33)) - e0 * Hinv[0, 1] / Hinv[0, 0]
    assert c[1] == int(np.clip(np.rint(np.float32(w1) / np.float32(s)), -8, 7)) and not c[2:].any()
    # a case where the feedback changes the code: rounding alone gives 3, the corrected weight rounds to 4
    R[0, 0], R[1, 0] = 0.70, 0.349
    R[2, 0] = 0.0
    H2 = np.eye(K)
    H2[0, 1] = H2[1, 0] = -0.9
    R[0, 0] = 0.655                                                  # e0 = 0.655 - 7 * (0.7/7)?  scale follows the absmax
    qw2, sw2 = oracle.gptq_quantize(R, H2, damp=0.0)
    c2, s2 = synth.unpack_int4(qw2)[0], float(sw2[0, 0])
    e0 = float(np.float32(0.655)) - c2[0] * s2
    Hi = np.linalg.inv(H2[:2, :2])
    w1 = float(np.float32(0.349)) - e0 * Hi[0, 1] / Hi[0, 0]
    assert c2[1] == int(np.clip(np.rint(np.float32(w1) / np.float32(s2)), -8, 7))


def test_objective_not_above_round_to_nearest():
    xb, il, H = correlated_hessian(3, 2000, 256)
    rng = np.random.default_rng(4)
    R = (rng.standard_normal((256, 64)) * 0.02).astype(np.float32)
    qg, sg = oracle.gptq_quantize(R, H, damp=0.01)
    qr, sr = synth.rtn_int4_weight(R)
    og, orr = oracle.gptq_objective(R, H, qg, sg), oracle.gptq_objective(R, H, qr, sr)
    assert og < 0.8 * orr, (og, orr)
    # and the objective is what it says: the output error on the calibration tokens
    xs = synth.bf16_bits_to_f32(xb).astype(np.float64)
    Rq = synth.unpack_int4(qg).T.astype(np.float64) * np.repeat(sg.astype(np.float64), 64, axis=0)
    assert abs(np.linalg.norm(xs @ (R - Rq)) ** 2 - og) <= 1e-9 * og


def test_dead_channel_and_damping():
    _, _, H = correlated_hessian(5, 300, 128)
    H[7, :] = 0.0
    H[:, 7] = 0.0
    R = (np.random.default_rng(6).standard_normal((128, 32)) * 0.02).astype(np.float32)
    qw, sw = oracle.gptq_quantize(R, H)
    assert not synth.unpack_int4(qw)[:, 7].any()                     # the unexcited input channel carries no weight


# ------------------------------------------------------------------------------------------------ GPU
@pytest.fixture(scope="module")
def svdq():
    import torch

    import paper_2605_27003_amd as m
    m.load_library(build_if_missing=False)
    assert torch.cuda.is_available()
    return m


@pytest.mark.gpu
@pytest.mark.parametrize("K,N,M", [(256, 128, 1500), (512, 256, 3000), (64, 128, 200), (320, 200, 1200)])
def test_gpu_gptq_bit_exact(svdq, K, N, M):
    import torch

    from tests.helpers import dev
    xb, il, H = correlated_hessian(10 + K, M, K)
    il = (np.random.default_rng(K).random(K).astype(np.float32) + 0.5)
    H = oracle.gptq_hessian(xb, il)
    Hg = svdq.gptq_hessian(dev(xb), dev(il))
    torch.cuda.synchronize()
    assert np.abs(Hg.cpu().numpy() - H).max() <= 1e-12 * np.abs(H).max()     # same sum, different order
    R = (np.random.default_rng(K + 1).standard_normal((K, N)) * 0.02).astype(np.float32)
    R[:, 3] = 0.0
    if K >= 128:
        H[9, :] = 0.0
        H[:, 9] = 0.0                                                         # a dead input channel
    qw, sw = svdq.gptq_quantize(dev(R), torch.from_numpy(H).cuda(), 0.01)
    torch.cuda.synchronize()
    oq, os_ = oracle.gptq_quantize(R, H, 0.01)
    assert np.array_equal(sw.cpu().numpy().view(np.uint32), os_.view(np.uint32))
    assert np.array_equal(qw.cpu().numpy(), oq)
    # and the product consumes it like any other canonical weight
    if N % 128 == 0:
        wp = svdq.pack_weight_e3m2(qw, sw)
        assert wp.numel() == svdq.packed_weight_e3m2_bytes(N, K)


@pytest.mark.gpu
def test_gpu_layer_error_drops_with_gptq_weights(svdq):
    """End to end on the GPU: the residual quantised by GPTQ on the layer's own calibration activations gives a
    smaller output error of the W4A4 layer than round-to-nearest (GPTQ with an identity Hessian) does."""
    import torch

    from tests.helpers import dev
    K, N, M = 512, 256, 4096
    xb, _, _ = correlated_hessian(77, M, K)
    il = torch.ones(K, device="cuda")
    x = dev(xb)
    R = (torch.randn(K, N, device="cuda", generator=torch.Generator("cuda").manual_seed(5)) * 0.02).float()
    H = svdq.gptq_hessian(x, il)
    H2 = svdq.gptq_hessian(x[: M // 2], il)
    svdq.gptq_hessian(x[M // 2:], il, H=H2)                                    # accumulation over calibration batches
    assert torch.allclose(H, H2, rtol=1e-12, atol=0)
    yref = (x.float() @ R).to(torch.bfloat16)
    act, _, _ = svdq.quantize_act_e3m2(x, il, 1.0, want_sx=False)
    errs = {}
    for name, (Hm, damp) in {"gptq": (H, 0.01), "rtn": (torch.eye(K, dtype=torch.float64, device="cuda"), 0.0)}.items():
        qw, sw = svdq.gptq_quantize(R, Hm, damp)
        y = svdq.linear_w4a4_e3m2(act, svdq.pack_weight_e3m2(qw, sw), N)
        errs[name] = float(svdq.sq_error(yref, y))
    torch.cuda.synchronize()
    assert errs["gptq"] < 0.75 * errs["rtn"], errs
