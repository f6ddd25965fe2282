"""GPU-vs-oracle parity of the MXFP4 variant through the C ABI.

Bar: E2M1 codes and E8M0 scale bytes bit-exact; y within relative Frobenius 2e-3 and max-abs 1e-2*rms(y)
of the oracle (helpers.check_y).  There are no integer accumulators in this variant: the matrix core
applies the block scales and accumulates in binary32 itself.
"""
import numpy as np
import pytest
import torch

from workloads import synth
from tests.helpers import check_y, dev, host_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def svdq():
    import paper_2605_27003_amd as m
    m.load_library(build_if_missing=False)
    assert torch.cuda.is_available()
    return m


class MxLayer:
    def __init__(self, svdq, L):
        self.L = L
        self.inv_lambda = dev(L.inv_lambda)
        self.L1 = dev(L.L1) if L.r else None
        self.L2 = dev(L.L2) if L.r else None
        self.bias = dev(L.bias)
        self.l1p = svdq.pack_lowrank_down(self.L1, self.inv_lambda) if L.r else None
        self.wp = svdq.pack_weight_mxfp4(dev(L.qw), dev(L.sw))


def small_layer(seed, M, K, N, r, outliers=3):
    x, cm = synth.make_x(seed, M, K, outlier_count=outliers, outlier_scale=30.0)
    return x, synth.make_layer(seed, K, N, r, cm, fmt="mxfp4")


def run_layer(svdq, oracle, x, L, rho, where):
    DL = MxLayer(svdq, L)
    M, K = x.shape
    qx, sx, h = svdq.quantize_act_mxfp4(dev(x), DL.inv_lambda, rho, DL.l1p, L.r)
    torch.cuda.synchronize()
    oq, os_ = oracle.quantize_act_mxfp4(x, L.inv_lambda, rho)
    gq, gs = svdq.mx_to_token_major(qx, sx, K)
    assert np.array_equal(gs.cpu().numpy(), os_), where + " scale bytes"
    assert np.array_equal(gq.cpu().numpy(), oq), where + " codes"
    if K % 128:                                            # the padding bytes of the odd last group are zero
        assert torch.all(sx[-1, :, :, 1] == 0)
    oh = None
    if L.r:
        oh = oracle.lowrank_down(x, L.inv_lambda, L.L1)
        hd = np.abs(h.cpu().numpy().astype(np.float64) - oh).max()
        assert hd <= 1e-4 * max(np.abs(oh).max(), 1e-30), (where, hd)
    y = svdq.linear_mxfp4(qx, sx, DL.wp, L.N, h, DL.L2, DL.bias)
    y32 = svdq.linear_mxfp4(qx, sx, DL.wp, L.N, h, DL.L2, DL.bias, out_dtype=torch.float32)
    torch.cuda.synchronize()
    orc = oracle.linear_mxfp4(oq, os_, L.qw, L.sw, oh, L.L2 if L.r else None, L.bias)
    check_y(host_bits(y), y32.cpu().numpy(), orc, where)
    return qx, sx, h, y


@pytest.mark.parametrize("rho", [1.0, 0.9, 0.6])
def test_c1_full_layer(svdq, oracle, rho):
    w = synth.workload(0, fmt="mxfp4")
    run_layer(svdq, oracle, w.x["x"], w.layers["e0/lin"], rho, f"c1 rho={rho}")


@pytest.mark.parametrize("M,K,N,r", [(333, 1024, 256, 32), (130, 192, 128, 16), (1, 64, 128, 16),
                                      (257, 448, 384, 0), (700, 2048, 128, 32),
                                      # few token tiles, many channel tiles: the channel-major tile order (both geometries)
                                      (333, 256, 2048, 32), (700, 192, 1152, 16)])
def test_ragged_shapes(svdq, oracle, M, K, N, r):
    x, L = small_layer(7, M, K, N, r)
    run_layer(svdq, oracle, x, L, 0.8, f"M={M} K={K} N={N} r={r}")


@pytest.mark.parametrize("M,K,N,r", [(1999, 640, 16384, 32), (2050, 1088, 16384, 16), (4100, 576, 8192, 0),
                                      (1999, 512, 16384, 32)])
def test_tile_walking_kernel_shapes(svdq, oracle, M, K, N, r):
    """Shapes with at least 512 tiles of 256 x 256 and K >= 576: the GEMM then runs as one block per CU that walks
    its tiles and stages each next tile's low-rank input in LDS.  Ragged last token tile, an odd group count, five
    to nine stages per tile, r = 32, 16 and none; the last shape (four stages) stays with one block per tile."""
    x, L = small_layer(11, M, K, N, r)
    run_layer(svdq, oracle, x, L, 0.8, f"tile-walking M={M} K={K} N={N} r={r}")


def test_tile_walking_kernel_without_bias(svdq, oracle):
    """The tile-walking GEMM with a low-rank branch and no bias, and with neither: its h transfers then read a
    substitute address and must leave the result alone."""
    M, K, N = 1100, 704, 32768
    for r in (32, 0):
        x, L = small_layer(13, M, K, N, r)
        DL = MxLayer(svdq, L)
        qx, sx, h = svdq.quantize_act_mxfp4(dev(x), DL.inv_lambda, 0.8, DL.l1p, r)
        y = svdq.linear_mxfp4(qx, sx, DL.wp, N, h, DL.L2 if r else None, None)
        y32 = svdq.linear_mxfp4(qx, sx, DL.wp, N, h, DL.L2 if r else None, None, out_dtype=torch.float32)
        torch.cuda.synchronize()
        oq, os_ = oracle.quantize_act_mxfp4(x, L.inv_lambda, 0.8)
        oh = oracle.lowrank_down(x, L.inv_lambda, L.L1) if r else None
        orc = oracle.linear_mxfp4(oq, os_, L.qw, L.sw, oh, L.L2 if r else None, None)
        check_y(host_bits(y), y32.cpu().numpy(), orc, f"tile-walking, no bias, r={r}")


def test_degenerate_blocks_and_ties(svdq, oracle):
    """All-zero rows and blocks, blocks below the scale range, the hand-worked tie vectors, saturation."""
    M, K, N, r = 40, 256, 128, 16
    x, L = small_layer(9, M, K, N, r)
    xf = synth.bf16_bits_to_f32(x).copy()
    xf[3, :] = 0.0
    xf[5, 32:64] = 0.0
    xf[6, 0:32] = 2.0 ** -126
    ties = [7.0, 0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 5.5, 6.0, -0.25, -0.75, -5.0, -7.0, -0.1, 0.0, 1.0, 1.5, 3.0]
    xf[8, 64:96] = 0.0
    xf[8, 64:64 + len(ties)] = ties
    L.inv_lambda[:] = 1.0
    L.lam[:] = 1.0
    qx, sx, h, y = run_layer(svdq, oracle, synth.to_bf16_bits(xf), L, 1.0, "degenerate")
    gq, gs = svdq.mx_to_token_major(qx, sx, K)
    gs = gs.cpu().numpy()
    assert gs[3].max() == 0 and gs[5, 1] == 0 and gs[6, 0] == 0 and gs[8, 2] == 127
    assert torch.isfinite(y.float()).all()


def test_determinism_and_guard_bands(svdq):
    M, K, N, r = 300, 1024, 256, 32
    x, L = small_layer(13, M, K, N, r)
    DL = MxLayer(svdq, L)
    xt = dev(x)
    pad = 64
    ns = (K // 64 + 1) // 2
    qbuf = torch.full((M * K // 2 + 2 * pad,), 0xAB, dtype=torch.uint8, device="cuda")
    sbuf = torch.full((ns * M * 4 + 2 * pad,), 0xCD, dtype=torch.uint8, device="cuda")
    hbuf = torch.full((M * r + 2 * pad,), -7.0, dtype=torch.float32, device="cuda")
    ybuf = torch.full((M * N + 2 * pad,), -7.0, dtype=torch.bfloat16, device="cuda")
    qx = qbuf[pad:-pad].view(K // 64, M, 32)
    sx = sbuf[pad:-pad].view(ns, M, 2, 2)
    h = hbuf[pad:-pad].view(M, r)
    y = ybuf[pad:-pad].view(M, N)
    svdq.quantize_act_mxfp4(xt, DL.inv_lambda, 0.8, DL.l1p, r, out=(qx, sx, h))
    svdq.linear_mxfp4(qx, sx, DL.wp, N, h, DL.L2, DL.bias, out=y)
    first = [t.clone() for t in (qx, sx, h, y)]
    svdq.quantize_act_mxfp4(xt, DL.inv_lambda, 0.8, DL.l1p, r, out=(qx, sx, h))
    svdq.linear_mxfp4(qx, sx, DL.wp, N, h, DL.L2, DL.bias, out=y)
    torch.cuda.synchronize()
    for a, b in zip(first, (qx, sx, h, y)):
        assert torch.equal(a, b)
    for buf, val in ((qbuf, 0xAB), (sbuf, 0xCD), (hbuf, -7.0), (ybuf, -7.0)):
        assert torch.all(buf[:pad] == val) and torch.all(buf[-pad:] == val)


# ---------------------------------------------------------------------------------------------
# full sizes, in the launch configuration bench.py times
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("idx", [1, 2, 3])
def test_full_size_configs(svdq, oracle, idx):
    """Codes and scale bytes over the WHOLE buffers (bit-exact), h on a row sample, y (bf16 and the pre-rounding
    binary32 value) on a seeded row sample: first 64, last 64 (ragged last tile), random rows."""
    from tests.helpers import rel_fro
    w = synth.workload(idx, fmt="mxfp4")
    L, x = w.layers["e0/lin"], w.x["x"]
    M, K = x.shape
    DL = MxLayer(svdq, L)
    rho = w.tables["e0"][0]
    qx, sx, h = svdq.quantize_act_mxfp4(dev(x), DL.inv_lambda, rho, DL.l1p, L.r)
    y16 = svdq.linear_mxfp4(qx, sx, DL.wp, L.N, h, DL.L2, DL.bias)
    torch.cuda.synchronize()
    fq, fs = oracle.quantize_act_mxfp4(x, L.inv_lambda, rho)
    gq, gs = svdq.mx_to_token_major(qx, sx, K)
    assert np.array_equal(gs.cpu().numpy(), fs), f"{w.name}: scale bytes (whole buffer)"
    assert np.array_equal(gq.cpu().numpy(), fq), f"{w.name}: codes (whole buffer)"
    del gq, gs
    S = synth.sample_rows(M, 1024 - 128, 40 + idx)
    St = torch.from_numpy(S).cuda()
    xs = np.ascontiguousarray(x[S])
    oh = oracle.lowrank_down(xs, L.inv_lambda, L.L1)
    assert rel_fro(h[St].cpu().numpy(), oh) <= 3e-5, f"{w.name}: h (row sample)"
    y32 = svdq.linear_mxfp4(qx, sx, DL.wp, L.N, h, DL.L2, DL.bias, out_dtype=torch.float32)
    torch.cuda.synchronize()
    orc = oracle.linear_mxfp4(np.ascontiguousarray(fq[S]), np.ascontiguousarray(fs[S]), L.qw, L.sw, oh, L.L2, L.bias)
    stats = check_y(host_bits(y16[St]), y32[St].cpu().numpy(), orc, w.name)
    print(f"{w.name} mxfp4 rho={rho}: whole-buffer codes/scales ok, y ok on {len(S)} rows {stats}", flush=True)


def test_resident_layer_object_mxfp4_and_gelu(svdq, oracle):
    """W4A4Linear with the MXFP4 container, and its gelu option (the down-projection of the feed-forward block taking the
    up-projection's pre-activation): outputs against the oracle's layer on the oracle's activated tensor."""
    from tests.helpers import rel_fro
    M, K, N, r = 150, 512, 256, 32
    x, _ = synth.make_x(33, M, K, outlier_count=3, outlier_scale=8.0, sigma=1.5)
    xg = oracle.gelu_tanh_bf16(x)
    cm = np.maximum(np.abs(synth.bf16_bits_to_f32(xg)).max(axis=0), 1e-3).astype(np.float32)
    L = synth.make_layer(33, K, N, r, cm, fmt="mxfp4")
    lin = svdq.W4A4Linear(dev(L.inv_lambda), dev(L.L1), dev(L.L2), dev(L.qw), dev(L.sw), dev(L.bias), container="mxfp4")
    oh = oracle.lowrank_down(xg, L.inv_lambda, L.L1)
    oq, os_ = oracle.quantize_act_mxfp4(xg, L.inv_lambda, 0.9)
    want = oracle.linear_mxfp4(oq, os_, L.qw, L.sw, oh, L.L2, L.bias)["y64"]
    for y in (lin.forward(dev(x), 0.9, gelu=True), lin.forward(dev(xg), 0.9)):
        torch.cuda.synchronize()
        assert rel_fro(synth.bf16_bits_to_f32(host_bits(y)).astype(np.float64), want) <= 2e-3
    ptr = y.data_ptr()
    assert lin.forward(dev(xg), 0.9).data_ptr() == ptr               # buffers are reused for a repeated shape
