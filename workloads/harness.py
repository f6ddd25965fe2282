"""Host <-> device plumbing and the output bar, shared by the GPU tests, bench.py and the smoke run.

Holds none of the layer's arithmetic: uploads of numpy arrays, a packed device copy of a synth.Layer made through
the library's own packers, and the comparison of a GPU output against values an oracle computed elsewhere.
"""
import numpy as np
import torch

from workloads import synth


def dev(a):
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
    # tighter than the stated bar: what the arithmetic should give.  The int8 GEMM adds 2.25*S per group to the
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
