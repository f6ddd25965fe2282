"""Benchmark of the W4A4 SVDQuant-style linear hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input:
the fused quantise kernel (smooth, absmax, clipped int4 quantise/pack, x^ L1)
followed by the W4A4 GEMM with its fused low-rank/bias/bf16 epilogue, on the
Wan2.2-shaped attention output projection (M=32760, K=N=5120, r=32); the
clipping ratio cycles through the layer's four timestep bins.  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0      # MI355X dense int8 matrix peak
HBM_PEAK_GBS = 8000.0             # MI355X HBM3E


def measured_traffic(workload_name, kernel):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload (FETCH_SIZE + WRITE_SIZE,
    each scaled by what the counter reads for a copy of known size), or None when there is no summary."""
    import re
    path = os.path.join(ROOT, "profiles", f"{workload_name.split(':')[0]}_hbm_traffic.txt")
    try:
        text = open(path).read()
    except OSError:
        return None
    m = re.search(rf"^traffic_bytes_per_launch\s+{kernel}\s+(\d+)", text, re.M)
    return int(m.group(1)) if m else None


def cpu_baseline(w, L, rows, seed=7):
    """The CPU oracle as it stands, timed on a row sample (rows are independent, so the sample is exact)."""
    import numpy as np

    import oracle
    from workloads import synth
    x = w.x["x"]
    S = synth.sample_rows(x.shape[0], rows - 128, seed)
    xs = np.ascontiguousarray(x[S])
    rho = w.tables["e0"][0]
    t0 = time.perf_counter()
    oq, os_ = oracle.quantize_act(xs, L.inv_lambda, rho)
    oh = oracle.lowrank_down(xs, L.inv_lambda, L.L1)
    t1 = time.perf_counter()
    oracle.linear(oq, os_, L.qw, L.sw, oh, L.L2, L.bias, want=("ybf16",))
    t2 = time.perf_counter()
    n = len(S)
    ops = 2.0 * n * L.N * L.K
    bytes_q = n * (2 * L.K + L.K // 2 + 4 * L.K // 64 + 4 * L.r)
    return {"value": ops / (t2 - t0) / 1e12, "unit": "TOPS", "cores": oracle.hw_threads(), "kind": "oracle",
            "sample": f"{n} of {x.shape[0]} token rows x full N={L.N} x full K={L.K} (quantize+lowrank {t1 - t0:.2f}s, "
                      f"linear {t2 - t1:.2f}s)",
            "quantize_GBs": bytes_q / (t1 - t0) / 1e9, "seconds": t2 - t0}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=50,
                    help="untimed steps; the clocks need some tens of launches after idle to settle")
    ap.add_argument("--workload", type=int, default=1, help="index into the five configurations (default: the metric's)")
    ap.add_argument("--cpu-rows", type=int, default=12288, help="token rows of the CPU-oracle baseline sample (0 = skip)")
    ap.add_argument("--xsets", type=int, default=3, help="input buffer sets rotated so caches cannot hold the working set")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; the path shards by token rows with no exchange step "
              "(see DESIGN.md), so --gpus N>1 is not implemented", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2605_27003_amd as svdq
    from tests.helpers import dev
    from workloads import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    svdq.load_library(build_if_missing=False)

    w = synth.workload(args.workload)
    lname = sorted(w.layers)[0]
    L = w.layers[lname]
    xname = w.inputs_of[lname.split("/")[1]]
    table = w.tables[lname.split("/")[0]]
    M, K, N, r = w.M, L.K, L.N, L.r

    lin = svdq.W4A4Linear(dev(L.inv_lambda), dev(L.L1), dev(L.L2), dev(L.qw), dev(L.sw), dev(L.bias))
    x0 = dev(w.x[xname])
    xs = [x0] + [x0.roll(17 * (i + 1), dims=0).contiguous() for i in range(args.xsets - 1)]
    qx, sx, h, y = lin.buffers(M, x0.device)
    ysets = [y] + [torch.empty_like(y) for _ in range(args.xsets - 1)]

    def step(i, ev=None):
        rho = table[i % len(table)]
        if ev:
            ev[0].record()
        svdq.quantize_act(xs[i % len(xs)], lin.inv_lambda, rho, lin.l1_packed, r, out=(qx, sx, h))
        if ev:
            ev[1].record()
        svdq.linear_w4a4(qx, sx, lin.w_packed, N, h, lin.L2, lin.bias, out=ysets[i % len(ysets)])
        if ev:
            ev[2].record()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, events[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_step = (t1 - t0) * 1e3 / args.steps
    tq = np.array([e[0].elapsed_time(e[1]) for e in events])          # ms, kernel (a)
    tg = np.array([e[1].elapsed_time(e[2]) for e in events])          # ms, kernels (b)+(c)
    ops = 2.0 * M * N * K
    bytes_q = M * (2 * K + K // 2 + 4 * K // 64 + 4 * r)              # read x, write codes, scales, h
    gemm_tops = ops / (tg.mean() * 1e-3) / 1e12
    quant_gbs = bytes_q / (tq.mean() * 1e-3) / 1e9

    out = {
        "metric": "W4A4 SVDQuant linear effective TOPS + % int8-MFMA peak; quantize pass GB/s",
        "value": ops / (ms_step * 1e-3) / 1e12, "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int4 x int4 -> int32 (int8 MFMA), fp32 dequant, bf16 out", "data": "synthetic",
        "config": {"workload": f"{w.name}: M={M} K={K} N={N} r={r} group=64, rho per timestep bin {table}",
                   "step": "svdq_quantize_act + svdq_linear_w4a4", "input_sets": len(xs)},
        "roofline": {"kernel": "svdq_linear_w4a4 (gemm_kernel)", "bound": "mfma",
                     "achieved": gemm_tops, "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                     "frac": gemm_tops / INT8_MFMA_PEAK_TOPS,
                     "traffic": measured_traffic(w.name, "gemm_kernel"),
                     "avg_ms": float(tg.mean()), "min_ms": float(tg.min())},
        "roofline_quantize": {"kernel": "svdq_quantize_act (quantize_kernel)", "bound": "hbm",
                              "achieved": quant_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": quant_gbs / HBM_PEAK_GBS,
                              "traffic": measured_traffic(w.name, "quantize_kernel"),
                              "algorithmic_bytes": bytes_q, "avg_ms": float(tq.mean()), "min_ms": float(tq.min())},
    }
    del xs, ysets
    if args.cpu_rows > 0:
        out["cpu_baseline"] = cpu_baseline(w, L, args.cpu_rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
