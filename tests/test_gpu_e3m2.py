"""GPU-vs-oracle parity of the E3M2-container execution of the int4 layer, through the C ABI.

The arithmetic is the int4 path's (eq. 3, 5, 7, 8, 11): the oracle functions and the bar are the same
(codes, scales and integer group sums bit-exact; y within relative Frobenius 2e-3 and max-abs 1e-2 rms).
The activation operand buffer is decoded on the host from the layout stated in include/svdq.h, by code that
shares nothing with the library, and the library's own unpack kernel is checked against that.
"""
import numpy as np
import pytest
import torch

from workloads import synth
from tests.helpers import (DeviceLayer, check_y, dev, host_bits, pack_act_e3m2_np, rel_fro, unpack_act_e3m2_np)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def svdq():
    import paper_2605_27003_amd as m
    m.load_library(build_if_missing=False)
    assert torch.cuda.is_available()
    return m


def small_layer(seed, M, K, N, r, outliers=3):
    x, cm = synth.make_x(seed, M, K, outlier_count=outliers, outlier_scale=30.0)
    return x, synth.make_layer(seed, K, N, r, cm)


def check_quant(svdq, oracle, x_bits, L, DL, rho, where):
    """Quantise on the GPU; codes, scales, scale pieces and h against the oracle.  Returns what the GEMM needs."""
    M, K = x_bits.shape
    act, sx, h = svdq.quantize_act_e3m2(dev(x_bits), DL.inv_lambda, rho, DL.l1p, L.r)
    torch.cuda.synchronize()
    oq, os_ = oracle.quantize_act(x_bits, L.inv_lambda, rho)
    codes, sxp = unpack_act_e3m2_np(act.buf.cpu().numpy(), M, K)
    assert np.array_equal(codes, synth.unpack_int4(oq)), where + " codes"
    assert np.array_equal(sx.cpu().numpy().T.view(np.uint32), os_.view(np.uint32)), where + " scales"
    # the two bf16 pieces stored for the scale-product instruction: hi = RNE(s), lo = RNE(s - hi)
    hi = synth.to_bf16_bits(os_)
    lo = synth.to_bf16_bits((os_ - synth.bf16_bits_to_f32(hi)).astype(np.float32))
    assert np.array_equal(sxp, hi.astype(np.uint32) | (lo.astype(np.uint32) << 16)), where + " scale pieces"
    # the library's own conversion back to nibbles
    qn = svdq.unpack_act_e3m2(act)
    assert np.array_equal(qn.permute(1, 0, 2).reshape(M, K // 2).cpu().numpy(), oq), where + " unpack"
    oh = None
    if L.r:
        oh = oracle.lowrank_down(x_bits, L.inv_lambda, L.L1)
        hg = h.cpu().numpy().astype(np.float64)
        assert rel_fro(hg, oh) <= 3e-5 and np.abs(hg - oh).max() <= 2e-4 * np.sqrt(np.mean(oh ** 2)), where
    return act, h, oq, os_, oh


def check_layer(svdq, oracle, x, L, rho, where, acc_rows=None):
    M = x.shape[0]
    DL = DeviceLayer(L)
    act, h, oq, os_, oh = check_quant(svdq, oracle, x, L, DL, rho, where)
    m0 = 0 if acc_rows is None else max(0, M - acc_rows)
    acc = svdq.debug_group_acc_e3m2(act, DL.wp6, L.N, m0, M - m0).cpu().numpy()
    assert np.array_equal(acc, oracle.group_acc(oq[m0:], L.qw)), where + " group sums"
    y16 = svdq.linear_w4a4_e3m2(act, DL.wp6, L.N, h, DL.L2, DL.bias)
    y32 = svdq.linear_w4a4_e3m2(act, DL.wp6, L.N, h, DL.L2, DL.bias, out_dtype=torch.float32)
    torch.cuda.synchronize()
    orc = oracle.linear(oq, os_, L.qw, L.sw, oh, L.L2 if L.r else None, L.bias)
    stats = check_y(host_bits(y16), y32.cpu().numpy(), orc, where)
    # no offset is carried in the accumulator here: the binary32 path is limited by the 16-bit scale pieces
    assert stats["rel_fro_f32"] <= 5e-5, (where, stats)
    return DL, act, h, y16


@pytest.mark.parametrize("rho", [1.0, 0.9, 0.6])
def test_c1_full_layer(svdq, oracle, rho):
    w = synth.workload(0)
    check_layer(svdq, oracle, w.x["x"], w.layers["e0/lin"], rho, f"e3m2 c1 rho={rho}")


@pytest.mark.parametrize("M,K,N,r", [(333, 1024, 256, 32), (130, 192, 128, 16), (1, 64, 128, 16), (2, 128, 128, 0),
                                     (3, 320, 128, 32), (127, 5120, 384, 32), (200, 2048, 128, 0), (261, 256, 256, 16),
                                     # few token tiles, many channel tiles: the channel-major tile order
                                     (333, 256, 1024, 32), (1200, 192, 2048, 16)])
def test_ragged_shapes(svdq, oracle, M, K, N, r):
    """Token counts around the row padding of the operand buffer (multiples of 4) and the 128-token tile, group
    counts below, at and above the depth of the staging ring (1, 2, 3, 4, 5, 16, 32, 80 groups)."""
    x, L = small_layer(7 + M, M, K, N, r)
    check_layer(svdq, oracle, x, L, 0.8, f"e3m2 M{M} K{K} N{N} r{r}", acc_rows=70)


def test_maximum_k(svdq, oracle):
    M, K, N, r = 70, 16384, 128, 16
    x, L = small_layer(19, M, K, N, r, outliers=5)
    check_layer(svdq, oracle, x, L, 0.9, "e3m2 max K", acc_rows=70)


def test_same_result_as_nibble_path(svdq):
    """Both executions hold the same codes and scales; their outputs differ only in binary32 rounding order."""
    M, K, N, r = 300, 1024, 256, 32
    x, L = small_layer(23, M, K, N, r)
    DL = DeviceLayer(L)
    xt = dev(x)
    qx, sx, h = svdq.quantize_act(xt, DL.inv_lambda, 0.8, DL.l1p, r)
    act, sx6, h6 = svdq.quantize_act_e3m2(xt, DL.inv_lambda, 0.8, DL.l1p, r)
    assert torch.equal(svdq.unpack_act_e3m2(act), qx) and torch.equal(sx, sx6) and torch.equal(h, h6)
    a4 = svdq.debug_group_acc(qx, DL.wp, N, 0, M)
    a6 = svdq.debug_group_acc_e3m2(act, DL.wp6, N, 0, M)
    assert torch.equal(a4, a6)
    y4 = svdq.linear_w4a4(qx, sx, DL.wp, N, h, DL.L2, DL.bias, out_dtype=torch.float32)
    y6 = svdq.linear_w4a4_e3m2(act, DL.wp6, N, h, DL.L2, DL.bias, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert rel_fro(y6.cpu().numpy(), y4.cpu().numpy()) <= 3e-4
    # sx output is optional
    act2, none, _ = svdq.quantize_act_e3m2(xt, DL.inv_lambda, 0.8, DL.l1p, r, want_sx=False)
    assert none is None and torch.equal(act2.buf[: act.buf.numel()], act.buf)


def test_degenerate_groups_and_ties(svdq, oracle):
    """All-zero rows and groups, a denormal group, the hand-worked tie vectors, codes at both range ends."""
    K = 256
    x = np.zeros((6, K), np.float32)
    x[1, 64:128] = np.linspace(-3, 3, 64)
    x[2, :64] = 1e-39
    ties = [14.0, 0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, 6.5, 7.5, 8.0, -7.5, -8.5, -9.0, -14.0, 0.25, 0.75, -0.75]
    x[3, : len(ties)] = ties
    x[4] = np.random.default_rng(0).standard_normal(K) * 100
    x[5, ::64] = 3e38
    xb = synth.to_bf16_bits(x)
    L = synth.make_layer(11, K, 128, 16, np.ones(K, np.float32))
    L.inv_lambda[:] = 1.0
    DL = DeviceLayer(L)
    for rho in (0.5, 1.0):
        check_quant(svdq, oracle, xb, L, DL, rho, f"degenerate rho={rho}")


def test_extreme_codes_from_a_hand_made_buffer(svdq, oracle):
    """Every code -8 on both sides: each group sum is 4096, the largest the path can see, and exact in the
    binary32 accumulator of the FP6 instruction.  The operand buffer is written by the host-side packer."""
    M, K, N = 131, 256, 128
    codes = np.full((M, K), -8, np.int64)
    codes[5] = 7
    codes[6, ::2] = 0
    qx = synth.pack_int4(codes)
    qw = np.full((N, K // 2), 0x88, np.uint8)
    qw[1::2] = 0x77                                             # rows of +7
    sw = np.ones((K // 64, N), np.float32)
    sx = np.ones((M, K // 64), np.float32)
    sx[7] = 0.0                                                 # dead groups
    wp = svdq.pack_weight_e3m2(dev(qw), dev(sw))
    act = svdq.ActE3M2(dev(pack_act_e3m2_np(codes, sx)), M, K)
    acc = svdq.debug_group_acc_e3m2(act, wp, N, 0, M).cpu().numpy()
    assert np.array_equal(acc, oracle.group_acc(qx, qw))
    assert acc.max() == 4096 and acc.min() == -3584
    y = svdq.linear_w4a4_e3m2(act, wp, N, out_dtype=torch.float32).cpu().numpy()
    want = oracle.linear(qx, sx, qw, sw)["y64"]
    assert np.array_equal(y.astype(np.float64), want)


def test_quantise_buffer_equals_host_packer(svdq, oracle):
    """Byte for byte (after mapping the hardware's negative zero to zero) the kernel's buffer is the documented
    layout of the oracle's codes and scales; padding rows are left alone."""
    M, K = 77, 320
    x, L = small_layer(29, M, K, 128, 0)
    DL = DeviceLayer(L)
    n = svdq.act_e3m2_bytes(M, K)
    buf = torch.full((n + 128,), 0xAB, dtype=torch.uint8, device="cuda")
    act = svdq.ActE3M2(buf[64: 64 + n], M, K)
    svdq.quantize_act_e3m2(dev(x), DL.inv_lambda, 0.9, out=(act, None, None))
    torch.cuda.synchronize()
    oq, os_ = oracle.quantize_act(x, L.inv_lambda, 0.9)
    want = pack_act_e3m2_np(synth.unpack_int4(oq), os_).reshape(K // 64, -1)
    got = act.buf.cpu().numpy().reshape(K // 64, -1)
    Mp = (M + 3) // 4 * 4
    for g in range(K // 64):
        assert np.array_equal(got[g, Mp * 32 + M * 8: Mp * 32 + Mp * 8], np.full((Mp - M) * 8, 0xAB, np.uint8))
        assert np.array_equal(got[g, Mp * 48 + M * 8:], np.full((Mp - M) * 8, 0xAB, np.uint8))
        assert np.array_equal(got[g, Mp * 48: Mp * 48 + M * 8], want[g, Mp * 48: Mp * 48 + M * 8])
    gc, _ = unpack_act_e3m2_np(got.reshape(-1), M, K)
    assert np.array_equal(gc, synth.unpack_int4(oq))
    assert torch.all(buf[:64] == 0xAB) and torch.all(buf[64 + n:] == 0xAB)


def test_strided_output_determinism_and_guard_bands(svdq):
    M, K, N, r = 200, 1024, 256, 32
    x, L = small_layer(13, M, K, N, r)
    DL = DeviceLayer(L)
    xt = dev(x)
    act, _, h = svdq.quantize_act_e3m2(xt, DL.inv_lambda, 0.8, DL.l1p, r, want_sx=False)
    ybuf = torch.full((M + 2, N + 24), 7.0, dtype=torch.bfloat16, device="cuda")
    y = svdq.linear_w4a4_e3m2(act, DL.wp6, N, h, DL.L2, DL.bias, out=ybuf[1:-1, :N])
    first = y.clone()
    act2, _, h2 = svdq.quantize_act_e3m2(xt, DL.inv_lambda, 0.8, DL.l1p, r, want_sx=False)
    svdq.linear_w4a4_e3m2(act2, DL.wp6, N, h2, DL.L2, DL.bias, out=ybuf[1:-1, :N])
    torch.cuda.synchronize()
    assert torch.equal(first, y) and torch.equal(act.buf, act2.buf)
    assert torch.all(ybuf[:, N:] == 7.0) and torch.all(ybuf[0] == 7.0) and torch.all(ybuf[-1] == 7.0)
    y_contig = svdq.linear_w4a4_e3m2(act, DL.wp6, N, h, DL.L2, DL.bias)
    assert torch.equal(y_contig, y)


def test_argument_errors(svdq):
    act = svdq.ActE3M2(torch.zeros(svdq.act_e3m2_bytes(8, 64), dtype=torch.uint8, device="cuda"), 8, 64)
    wp = torch.zeros(svdq.packed_weight_e3m2_bytes(128, 64), dtype=torch.uint8, device="cuda")
    with pytest.raises(svdq.SvdqError):
        svdq.linear_w4a4_e3m2(act, wp, 100)                      # N not a multiple of 128
    assert svdq.packed_weight_e3m2_bytes(100, 64) == 0 and svdq.act_e3m2_bytes(8, 65) == 0
    x = torch.zeros((8, 64), dtype=torch.bfloat16, device="cuda")
    il = torch.ones(64, device="cuda")
    with pytest.raises(svdq.SvdqError):
        svdq.quantize_act_e3m2(x, il, 1.5)                       # rho out of range
    with pytest.raises(svdq.SvdqError):
        svdq.debug_group_acc_e3m2(act, wp, 128, 4, 8)            # rows beyond M


@pytest.mark.parametrize("container", ["e3m2", "nibble"])
def test_resident_layer_object(svdq, oracle, container):
    """W4A4Linear (packed weights and reusable buffers behind forward()) gives the layer's output for both
    containers, reuses its buffers for a repeated shape and re-allocates for a new one."""
    M, K, N, r = 150, 512, 256, 32
    x, L = small_layer(31, M, K, N, r)
    lin = svdq.W4A4Linear(dev(L.inv_lambda), dev(L.L1), dev(L.L2), dev(L.qw), dev(L.sw), dev(L.bias), container=container)
    y = lin.forward(dev(x), 0.9)
    torch.cuda.synchronize()
    oq, os_ = oracle.quantize_act(x, L.inv_lambda, 0.9)
    orc = oracle.linear(oq, os_, L.qw, L.sw, oracle.lowrank_down(x, L.inv_lambda, L.L1), L.L2, L.bias)
    yb = synth.bf16_bits_to_f32(host_bits(y)).astype(np.float64)
    assert rel_fro(yb, orc["y64"]) <= 2e-3
    ptr = y.data_ptr()
    assert lin.forward(dev(x), 0.9).data_ptr() == ptr
    y2 = lin.forward(dev(x[:70]), 0.9)
    torch.cuda.synchronize()
    assert y2.shape == (70, N) and torch.equal(y2, lin.forward(dev(x[:70]), 0.9))
    assert rel_fro(synth.bf16_bits_to_f32(host_bits(y2)).astype(np.float64), orc["y64"][:70]) <= 2e-3


def test_layers_with_resident_4bit_weights_share_one_staging_buffer(svdq, oracle):
    """The default residency of the E3M2 execution: every layer keeps the canonical 4-bit weights and expands them
    into ONE staging buffer right before its GEMM.  Two layers of different shapes used alternately give exactly the
    outputs of the same layers with their expanded weights resident."""
    layers = []
    for seed, (M, K, N, r) in enumerate([(150, 512, 256, 32), (150, 256, 384, 16)]):
        x, L = small_layer(40 + seed, M, K, N, r)
        args = (dev(L.inv_lambda), dev(L.L1), dev(L.L2), dev(L.qw), dev(L.sw), dev(L.bias))
        layers.append((dev(x), svdq.W4A4Linear(*args), svdq.W4A4Linear(*args, resident="packed")))
    assert layers[0][1].w_packed is None and layers[0][2].w_packed is not None
    for rep in range(2):
        for xd, w4, packed in layers:
            y = w4.forward(xd, 0.8).clone()
            assert torch.equal(y, packed.forward(xd, 0.8))
    torch.cuda.synchronize()
    from paper_2605_27003_amd import binding
    assert len(binding._staging) == 1
    (buf,) = binding._staging.values()
    assert buf.numel() == max(svdq.packed_weight_e3m2_bytes(256, 512), svdq.packed_weight_e3m2_bytes(384, 256))
