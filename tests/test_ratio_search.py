"""Timestep-bin clipping-ratio search (Sec. III-C): oracle pins on the CPU, GPU-vs-oracle parity on the GPU."""
import numpy as np
import pytest

from workloads import synth

CANDIDATES = [0.6, 0.7, 0.8, 0.9, 1.0]


def bf16(a):
    return synth.to_bf16_bits(np.asarray(a, np.float32))


def f32(b):
    return synth.bf16_bits_to_f32(np.asarray(b, np.uint16))


def calibration_set(seed, M, K, N, r, nsteps, nbins, fmt="int4"):
    """A small layer and `nsteps` calibration steps whose dynamic range shrinks along the trajectory (early steps
    carry stronger outlier channels, as Sec. III-C describes); the full-precision output is x W + b."""
    x0, cm = synth.make_x(seed, M, K, outlier_count=4, outlier_scale=40.0)
    L = synth.make_layer(seed, K, N, r, cm, keep_dense=True, fmt=fmt)
    rng = np.random.default_rng(seed)
    xs, yrefs, bins = [], [], []
    for t in range(nsteps):
        xf = f32(np.roll(x0, 7 * t, axis=0)).copy()
        out_ch = rng.permutation(K)[:4]
        xf[:, out_ch] *= np.float32(1.0 + 3.0 * (nsteps - 1 - t) / max(nsteps - 1, 1))
        xb = bf16(xf)
        xs.append(xb)
        yrefs.append(bf16((f32(xb).astype(np.float64) @ L.W.astype(np.float64) + L.bias).astype(np.float32)))
        bins.append(t * nbins // nsteps)
    return L, xs, yrefs, bins


# ---------------------------------------------------------------------------------- CPU pins
def test_sq_error_matches_numpy(oracle):
    rng = np.random.default_rng(1)
    a, b = bf16(rng.standard_normal((37, 64))), bf16(rng.standard_normal((37, 64)))
    want = float(((f32(a).astype(np.float64) - f32(b).astype(np.float64)) ** 2).sum())
    assert abs(oracle.sq_error(a, b) - want) <= 1e-12 * want


def test_search_picks_rho_one_when_everything_lies_on_the_grid(oracle):
    """Inputs exactly on the int4 grid of rho = 1 and weights that ARE their dequantised codes: the quantised
    layer at rho = 1 reproduces the full-precision output, any smaller ratio clips the +-7 entries."""
    rng = np.random.default_rng(3)
    M, K, N = 24, 128, 128
    q = rng.integers(-7, 8, size=(M, K)).astype(np.float32)
    q[:, ::64] = 7.0
    x = bf16(q * np.float32(0.125))
    cm = np.abs(f32(x)).max(axis=0)
    L = synth.make_layer(5, K, N, 0, cm, keep_dense=True)
    L.inv_lambda[:] = 1.0
    L.lam[:] = 1.0
    Wdq = (synth.unpack_int4(L.qw).astype(np.float64).T *
           np.repeat(L.sw.astype(np.float64), 64, axis=0))                       # [K,N] = codes * scales
    yref = bf16((f32(x).astype(np.float64) @ Wdq + L.bias).astype(np.float32))
    table, err = oracle.search_clipping_ratios(L, [x, x], [yref, yref], [0, 1], 2, CANDIDATES)
    assert table == [1.0, 1.0]
    assert err[0, -1] == 0.0 and np.all(err[:, :-1] > 0)


def test_search_table_is_the_per_bin_argmin_and_differs_between_bins(oracle):
    L, xs, yrefs, bins = calibration_set(11, 64, 256, 128, 16, nsteps=4, nbins=2)
    table, err = oracle.search_clipping_ratios(L, xs, yrefs, bins, 2, CANDIDATES)
    assert err.shape == (2, 5) and np.all(err > 0)
    assert table == [CANDIDATES[i] for i in err.argmin(axis=1)]
    # the objective really depends on the ratio: best and worst candidate differ clearly
    assert np.all(err.max(axis=1) > 1.02 * err.min(axis=1))


# ---------------------------------------------------------------------------------- GPU parity
@pytest.mark.gpu
@pytest.mark.parametrize("fmt", ["int4", "mxfp4"])
def test_gpu_search_matches_oracle(oracle, fmt):
    import torch
    import paper_2605_27003_amd as svdq
    from tests.helpers import dev
    svdq.load_library(build_if_missing=False)
    M, K, N, r, nsteps, nbins = 256, 512, 256, 16, 8, 4
    L, xs, yrefs, bins = calibration_set(21, M, K, N, r, nsteps, nbins, fmt=fmt)
    inv_lambda, L2, bias = dev(L.inv_lambda), dev(L.L2), dev(L.bias)
    l1p = svdq.pack_lowrank_down(dev(L.L1), inv_lambda)
    if fmt == "int4":
        wp = svdq.pack_weight(dev(L.qw), dev(L.sw))
        def run(x, rho):
            qx, sx, h = svdq.quantize_act(x, inv_lambda, rho, l1p, r)
            return svdq.linear_w4a4(qx, sx, wp, N, h, L2, bias)
    else:
        wp = svdq.pack_weight_mxfp4(dev(L.qw), dev(L.sw))
        def run(x, rho):
            qx, sx, h = svdq.quantize_act_mxfp4(x, inv_lambda, rho, l1p, r)
            return svdq.linear_mxfp4(qx, sx, wp, N, h, L2, bias)
    table, err = svdq.search_clipping_ratios(run, [dev(x) for x in xs], [dev(y) for y in yrefs], bins, nbins, CANDIDATES)
    otable, oerr = oracle.search_clipping_ratios(L, xs, yrefs, bins, nbins, CANDIDATES, fmt=fmt)
    # the sums: bf16 outputs of the two sides differ in a small fraction of last bits, so compare with a tolerance
    assert np.allclose(err, oerr, rtol=5e-3), (err, oerr)
    # the arg-min: must agree wherever the oracle's best candidate wins by more than that tolerance
    for b in range(nbins):
        srt = np.sort(oerr[b])
        if srt[1] > 1.01 * srt[0]:
            assert table[b] == otable[b], (b, err[b], oerr[b])
    # the reduction kernel alone: exact same inputs on both sides
    y = run(dev(xs[0]), 0.8)
    e = svdq.sq_error(dev(yrefs[0]), y)
    torch.cuda.synchronize()
    want = oracle.sq_error(yrefs[0], y.cpu().view(torch.int16).numpy().view(np.uint16))
    # the kernel adds each 8-element chunk in binary32 (relative error <= 8 * 2^-24) and the chunks in binary64
    assert abs(float(e[0]) - want) <= 8 * 2.0 ** -24 * want
    print(f"{fmt}: table {table} (oracle {otable})")
