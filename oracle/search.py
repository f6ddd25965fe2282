"""Oracle of the timestep-bin clipping-ratio search (Sec. III-C, the arg-min over the candidate set).

TEST INFRASTRUCTURE, NOT PRODUCT.  Plain loop over calibration steps and candidates around the C++ oracle's layer
and its squared-error sum; numpy only adds the per-bin sums and takes the arg-min.
"""
import numpy as np

from . import linear, linear_mxfp4, lowrank_down, quantize_act, quantize_act_mxfp4, sq_error


def search_clipping_ratios(layer, xs, y_refs, bins, nbins, candidates, fmt="int4"):
    """For every timestep bin: the candidate ratio with the smallest summed squared reconstruction error of the
    quantised layer over the bin's calibration steps.  `layer` has inv_lambda, L1, L2, qw, sw, bias (numpy);
    xs[i] / y_refs[i] are bf16 bit arrays.  Returns (table, err [nbins][len(candidates)])."""
    err = np.zeros((nbins, len(candidates)), np.float64)
    for x, yr, b in zip(xs, y_refs, bins):
        h = lowrank_down(x, layer.inv_lambda, layer.L1) if layer.r else None
        for ci, rho in enumerate(candidates):
            if fmt == "mxfp4":
                qx, sx = quantize_act_mxfp4(x, layer.inv_lambda, rho)
                y = linear_mxfp4(qx, sx, layer.qw, layer.sw, h, layer.L2 if layer.r else None, layer.bias, want=("ybf16",))
            else:
                qx, sx = quantize_act(x, layer.inv_lambda, rho)
                y = linear(qx, sx, layer.qw, layer.sw, h, layer.L2 if layer.r else None, layer.bias, want=("ybf16",))
            err[b, ci] += sq_error(yr, y["ybf16"])
    table = [float(candidates[int(i)]) for i in err.argmin(axis=1)]
    return table, err
