"""Benchmark of the W4A4 SVDQuant-style linear hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input:
the fused quantise kernel (smooth, absmax, clipped int4 quantise/pack, x^ L1)
followed by the W4A4 GEMM with its fused low-rank/bias/bf16 epilogue, on the
Wan2.2-shaped attention output projection (M=32760, K=N=5120, r=32); the
clipping ratio cycles through the layer's four timestep bins.  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line; its headline
fields are the int4 path, "mxfp4_variant" carries the same layer in the MXFP4
format and "context" a dense bf16 GEMM of the same shape.
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
    ap.add_argument("--skip-mxfp4", action="store_true", help="do not also time the MXFP4 variant of the layer")
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

    FP4_MFMA_PEAK_TFLOPS = 10100.0    # MI355X dense fp4 matrix peak

    def measure(fmt):
        """One pass of the hot path per step for the given 4-bit format; returns the timing record."""
        w = synth.workload(args.workload, fmt=fmt)
        lname = sorted(w.layers)[0]
        L = w.layers[lname]
        xname = w.inputs_of[lname.split("/")[1]]
        table = w.tables[lname.split("/")[0]]
        M, K, N, r = w.M, L.K, L.N, L.r
        inv_lambda, L2, bias = dev(L.inv_lambda), dev(L.L2), dev(L.bias)
        l1p = svdq.pack_lowrank_down(dev(L.L1), inv_lambda)
        x0 = dev(w.x[xname])
        xs = [x0] + [x0.roll(17 * (i + 1), dims=0).contiguous() for i in range(args.xsets - 1)]
        ysets = [torch.empty((M, N), dtype=torch.bfloat16, device=x0.device) for _ in range(args.xsets)]
        h = torch.empty((M, r), dtype=torch.float32, device=x0.device)
        qx = torch.empty((K // 64, M, 32), dtype=torch.uint8, device=x0.device)
        if fmt == "int4":
            wp = svdq.pack_weight(dev(L.qw), dev(L.sw))
            sx = torch.empty((K // 64, M), dtype=torch.float32, device=x0.device)
            quant, gemm = svdq.quantize_act, svdq.linear_w4a4
            scale_bytes = 4 * (K // 64)
        else:
            wp = svdq.pack_weight_mxfp4(dev(L.qw), dev(L.sw))
            sx = torch.empty(((K // 64 + 1) // 2, M, 2, 2), dtype=torch.uint8, device=x0.device)
            quant, gemm = svdq.quantize_act_mxfp4, svdq.linear_mxfp4
            scale_bytes = K // 32

        def step(i, ev=None):
            rho = table[i % len(table)]
            if ev:
                ev[0].record()
            quant(xs[i % len(xs)], inv_lambda, rho, l1p, r, out=(qx, sx, h))
            if ev:
                ev[1].record()
            gemm(qx, sx, wp, N, h, L2, bias, out=ysets[i % len(ysets)])
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
        # dense bf16 GEMM of the same shape from the vendor library: what the paper's BF16 baseline costs here
        wd = torch.empty((K, N), dtype=torch.bfloat16, device=x0.device).normal_()
        for _ in range(5):
            torch.matmul(xs[0], wd, out=ysets[0])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(20):
            torch.matmul(xs[i % len(xs)], wd, out=ysets[i % len(ysets)])
        e1.record()
        torch.cuda.synchronize()
        return dict(w=w, L=L, table=table, M=M, K=K, N=N, r=r, ms_step=ms_step, tq=tq, tg=tg, nx=len(xs),
                    ops=2.0 * M * N * K, bytes_q=M * (2 * K + K // 2 + scale_bytes + 4 * r),
                    bf16_ms=e0.elapsed_time(e1) / 20)

    def measure_block(fmt):
        """Workload with several linears (the 720p DiT block): one step = every linear's quantise pass and GEMM for the
        expert and clipping ratios of that denoising step, walking the 40-step schedule (expert switch included)."""
        w = synth.workload(args.workload, fmt=fmt)
        M = w.M
        xdev = {k: dev(v) for k, v in w.x.items()}
        per_expert = {}
        for ename in w.experts:
            lins = []
            for lin, inp in w.inputs_of.items():
                L = w.layers[f"{ename}/{lin}"]
                inv_lambda = dev(L.inv_lambda)
                rec = dict(L=L, x=xdev[inp], inv_lambda=inv_lambda, L2=dev(L.L2), bias=dev(L.bias),
                           l1p=svdq.pack_lowrank_down(dev(L.L1), inv_lambda),
                           wp=(svdq.pack_weight if fmt == "int4" else svdq.pack_weight_mxfp4)(dev(L.qw), dev(L.sw)))
                lins.append(rec)
            per_expert[ename] = lins
        bufs = {}
        for rec in per_expert[w.experts[0]]:
            K, N, r = rec["L"].K, rec["L"].N, rec["L"].r
            if (K, N) not in bufs:
                sx = (torch.empty((K // 64, M), dtype=torch.float32, device="cuda") if fmt == "int4"
                      else torch.empty(((K // 64 + 1) // 2, M, 2, 2), dtype=torch.uint8, device="cuda"))
                bufs[(K, N)] = (torch.empty((K // 64, M, 32), dtype=torch.uint8, device="cuda"), sx,
                                torch.empty((M, r), dtype=torch.float32, device="cuda"),
                                torch.empty((M, N), dtype=torch.bfloat16, device="cuda"))
        quant = svdq.quantize_act if fmt == "int4" else svdq.quantize_act_mxfp4
        gemm = svdq.linear_w4a4 if fmt == "int4" else svdq.linear_mxfp4

        def step(i, evs=None):
            t = i % w.nsteps
            e = 0 if t < w.switch_step else 1
            step0 = 0 if e == 0 else w.switch_step
            nst = w.switch_step if e == 0 else w.nsteps - w.switch_step
            rho = svdq.alpha_lookup(w.tables[w.experts[e]], t, step0, nst)
            for li, rec in enumerate(per_expert[w.experts[e]]):
                L = rec["L"]
                qx, sx, h, y = bufs[(L.K, L.N)]
                if evs:
                    evs[li][0].record()
                quant(rec["x"], rec["inv_lambda"], rho, rec["l1p"], L.r, out=(qx, sx, h))
                if evs:
                    evs[li][1].record()
                gemm(qx, sx, rec["wp"], L.N, h, rec["L2"], rec["bias"], out=y)
                if evs:
                    evs[li][2].record()

        nl = len(per_expert[w.experts[0]])
        for i in range(args.warmup):
            step(i)
        torch.cuda.synchronize()
        events = [[[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(nl)] for _ in range(args.steps)]
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i, events[i])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        tq = np.array([sum(e[0].elapsed_time(e[1]) for e in ev) for ev in events])
        tg = np.array([sum(e[1].elapsed_time(e[2]) for e in ev) for ev in events])
        ops = sum(2.0 * M * rec["L"].N * rec["L"].K for rec in per_expert[w.experts[0]])
        sb = (lambda K: 4 * (K // 64)) if fmt == "int4" else (lambda K: K // 32)
        bytes_q = sum(M * (2 * rec["L"].K + rec["L"].K // 2 + sb(rec["L"].K) + 4 * rec["L"].r) for rec in per_expert[w.experts[0]])
        return dict(w=w, M=M, ms_step=(t1 - t0) * 1e3 / args.steps, tq=tq, tg=tg, ops=ops, bytes_q=bytes_q, nl=nl)

    if args.workload == 4:
        recs = {"int4": measure_block("int4")}
        if not args.skip_mxfp4:
            recs["mxfp4"] = measure_block("mxfp4")
        B = recs["int4"]
        gt = B["ops"] / (B["tg"].mean() * 1e-3) / 1e12
        qg = B["bytes_q"] / (B["tq"].mean() * 1e-3) / 1e9
        out = {
            "metric": "W4A4 SVDQuant linear effective TOPS + % int8-MFMA peak; quantize pass GB/s",
            "value": B["ops"] / (B["ms_step"] * 1e-3) / 1e12, "unit": "TOPS",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": B["ms_step"],
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "int4 x int4 -> int32 (int8 MFMA), fp32 dequant, bf16 out", "data": "synthetic",
            "config": {"workload": f"{B['w'].name}: M={B['M']}, six linears (q, k, v, o 5120x5120; ffn_up 5120x13824; "
                                   f"ffn_down 13824x5120) r=32, two experts over a 40-step schedule, ratio per timestep bin",
                       "step": f"{B['nl']} x (svdq_quantize_act + svdq_linear_w4a4) = one DiT block-step"},
            "roofline": {"kernel": "svdq_linear_w4a4 (gemm_kernel), six launches", "bound": "mfma", "achieved": gt,
                         "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s", "frac": gt / INT8_MFMA_PEAK_TOPS, "traffic": None,
                         "avg_ms": float(B["tg"].mean()), "min_ms": float(B["tg"].min())},
            "roofline_quantize": {"kernel": "svdq_quantize_act (quantize_kernel), six launches", "bound": "hbm",
                                  "achieved": qg, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": qg / HBM_PEAK_GBS,
                                  "traffic": None, "algorithmic_bytes": B["bytes_q"],
                                  "avg_ms": float(B["tq"].mean()), "min_ms": float(B["tq"].min())},
        }
        if "mxfp4" in recs:
            X = recs["mxfp4"]
            g = X["ops"] / (X["tg"].mean() * 1e-3) / 1e12
            out["mxfp4_variant"] = {"value": X["ops"] / (X["ms_step"] * 1e-3) / 1e12, "unit": "TFLOP/s",
                                    "ms_per_step": X["ms_step"], "gemm_TFLOPs": g, "gemm_frac_of_fp4_peak": g / FP4_MFMA_PEAK_TFLOPS,
                                    "gemm_ms": float(X["tg"].mean()), "quantize_ms": float(X["tq"].mean())}
        print(json.dumps(out))
        return

    R = measure("int4")
    w, L, table, M, K, N, r = R["w"], R["L"], R["table"], R["M"], R["K"], R["N"], R["r"]
    ops, bytes_q, tq, tg, ms_step = R["ops"], R["bytes_q"], R["tq"], R["tg"], R["ms_step"]
    gemm_tops = ops / (tg.mean() * 1e-3) / 1e12
    quant_gbs = bytes_q / (tq.mean() * 1e-3) / 1e9

    out = {
        "metric": "W4A4 SVDQuant linear effective TOPS + % int8-MFMA peak; quantize pass GB/s",
        "value": ops / (ms_step * 1e-3) / 1e12, "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int4 x int4 -> int32 (int8 MFMA), fp32 dequant, bf16 out", "data": "synthetic",
        "config": {"workload": f"{w.name}: M={M} K={K} N={N} r={r} group=64, rho per timestep bin {table}",
                   "step": "svdq_quantize_act + svdq_linear_w4a4", "input_sets": R["nx"]},
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
        "context": {"bf16_dense_matmul_ms": R["bf16_ms"],
                    "note": "vendor-library bf16 GEMM of the same shape on the same GPU (the paper's BF16 baseline)"},
    }
    if not args.skip_mxfp4:
        X = measure("mxfp4")
        g = X["ops"] / (X["tg"].mean() * 1e-3) / 1e12
        q = X["bytes_q"] / (X["tq"].mean() * 1e-3) / 1e9
        out["mxfp4_variant"] = {
            "what": "same layer in the MXFP4 format of the paper's Table I on the block-scaled FP4 matrix instruction",
            "value": X["ops"] / (X["ms_step"] * 1e-3) / 1e12, "unit": "TFLOP/s", "ms_per_step": X["ms_step"],
            "roofline": {"kernel": "svdq_linear_mxfp4 (gemm_mx_kernel)", "bound": "mfma", "achieved": g,
                         "peak": FP4_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": g / FP4_MFMA_PEAK_TFLOPS,
                         "traffic": measured_traffic(w.name, "gemm_mx_kernel"),
                         "avg_ms": float(X["tg"].mean()), "min_ms": float(X["tg"].min())},
            "roofline_quantize": {"kernel": "svdq_quantize_act_mxfp4 (quantize_mx_kernel)", "bound": "hbm",
                                  "achieved": q, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": q / HBM_PEAK_GBS,
                                  "traffic": measured_traffic(w.name, "quantize_mx_kernel"),
                                  "algorithmic_bytes": X["bytes_q"], "avg_ms": float(X["tq"].mean()),
                                  "min_ms": float(X["tq"].min())},
            "speedup_vs_bf16_dense": X["bf16_ms"] / X["ms_step"]}
        del X
    if args.cpu_rows > 0:
        out["cpu_baseline"] = cpu_baseline(w, L, args.cpu_rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
