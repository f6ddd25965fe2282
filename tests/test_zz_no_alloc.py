"""The reduction of the clipping-ratio search through the entry point that allocates nothing (partial sums in the
library's static device array) against the entry point that takes a caller workspace: two calls in a row, the
second on a smaller input, results identical bit for bit and within the reduction's bound of the oracle."""
import ctypes

import numpy as np
import pytest

from workloads import synth


@pytest.mark.gpu
def test_sq_error_static_matches_workspace_entry_point(oracle):
    import torch
    import paper_2605_27003_amd as svdq
    from workloads.harness import dev
    lib = svdq.load_library(build_if_missing=False)
    rng = np.random.default_rng(5)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    ws = torch.empty(lib.svdq_sq_error_workspace_bytes() // 8, dtype=torch.float64, device="cuda")
    for M, N, ld in ((1537, 1024, 1032), (93, 256, 256)):          # the second call is smaller than the first
        a = synth.to_bf16_bits(rng.standard_normal((M, ld)).astype(np.float32))
        b = synth.to_bf16_bits(rng.standard_normal((M, ld)).astype(np.float32))
        ta, tb = dev(a), dev(b)
        want = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
        got = torch.full((1,), -2.0, dtype=torch.float64, device="cuda")
        print(f"sq_error_static case M={M} N={N} ld={ld}", flush=True)
        # raw C ABI: the existing entry point with a workspace, then the one without
        rc = lib.svdq_sq_error(ctypes.c_void_p(ta.data_ptr()), ld, ctypes.c_void_p(tb.data_ptr()), ld, M, N,
                               ctypes.c_void_p(ws.data_ptr()), ctypes.c_void_p(want.data_ptr()), stream)
        assert rc == 0
        rc = lib.svdq_sq_error_static(ctypes.c_void_p(ta.data_ptr()), ld, ctypes.c_void_p(tb.data_ptr()), ld, M, N,
                                      ctypes.c_void_p(got.data_ptr()), stream)
        assert rc == 0
        torch.cuda.synchronize()
        assert got.cpu().numpy().view(np.uint64)[0] == want.cpu().numpy().view(np.uint64)[0], (float(got[0]), float(want[0]))
        ref = oracle.sq_error(np.ascontiguousarray(a[:, :N]), np.ascontiguousarray(b[:, :N]))
        # each 8-element chunk is summed in binary32 (relative error <= 8 * 2^-24), the chunks in binary64
        assert abs(float(got[0]) - ref) <= 8 * 2.0 ** -24 * ref
    # M == 0 gives 0 without touching the inputs
    rc = lib.svdq_sq_error_static(ctypes.c_void_p(ta.data_ptr()), ld, ctypes.c_void_p(tb.data_ptr()), ld, 0, N,
                                  ctypes.c_void_p(got.data_ptr()), stream)
    assert rc == 0
    torch.cuda.synchronize()
    assert float(got[0]) == 0.0
    # the binding's wrapper of the same entry point
    assert float(svdq.sq_error_static(ta[:, :N], tb[:, :N])[0]) == float(want[0])
