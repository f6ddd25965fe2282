"""Benchmark of the W4A4 SVDQuant-style linear hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input:
the fused quantise kernel (smooth, absmax, clipped int4 quantise/pack, x^ L1)
followed by the W4A4 GEMM with its fused low-rank/bias/bf16 epilogue, on the
Wan2.2-shaped attention output projection (M=32760, K=N=5120, r=32); the
clipping ratio cycles through the layer's four timestep bins.  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line; its headline
fields are the int4 layer executed on the FP6 matrix cores (codes held as E3M2
fields, bit-identical integer arithmetic), "int4_nibble_variant" is the same
layer on 4-bit storage and the int8 matrix cores, "mxfp4_variant" the same
layer in the MXFP4 format and "context" a dense bf16 GEMM of the same shape.
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
FP6_MFMA_PEAK_TFLOPS = 10100.0    # MI355X dense fp6 / fp4 matrix peak
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
    ap.add_argument("--ffn-chain", action="store_true",
                    help="also time the feed-forward chain up-projection -> GELU -> down-projection, un-fused (three "
                         "kernels) and with the GEMM epilogue that emits the next layer's operands (two kernels)")
    ap.add_argument("--xsets", type=int, default=3, help="input buffer sets rotated so caches cannot hold the working set")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; the path shards by token rows with no exchange step "
              "so --gpus N>1 is not implemented", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2605_27003_amd as svdq
    from tests.helpers import dev
    from workloads import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    svdq.load_library(build_if_missing=False)

    FP4_MFMA_PEAK_TFLOPS = FP6_MFMA_PEAK_TFLOPS

    def kernels_of(fmt, K, M, device):
        """(weight packer, quantise call, GEMM call, activation buffers, scale bytes per token) of one execution:
        "e3m2" = int4 codes as E3M2 fields on the FP6 matrix cores, "int4" = 4-bit storage on the int8 matrix cores,
        "mxfp4" = the MXFP4 format."""
        if fmt == "e3m2":
            act = svdq.ActE3M2(torch.empty(svdq.act_e3m2_bytes(M, K), dtype=torch.uint8, device=device), M, K)
            return (svdq.pack_weight_e3m2,
                    lambda x, il, rho, l1p, r, h: svdq.quantize_act_e3m2(x, il, rho, l1p, r, out=(act, None, h)),
                    lambda wp, N, h, L2, b, y: svdq.linear_w4a4_e3m2(act, wp, N, h, L2, b, out=y), 4 * (K // 64))
        qx = torch.empty((K // 64, M, 32), dtype=torch.uint8, device=device)
        if fmt == "int4":
            sx = torch.empty((K // 64, M), dtype=torch.float32, device=device)
            return (svdq.pack_weight,
                    lambda x, il, rho, l1p, r, h: svdq.quantize_act(x, il, rho, l1p, r, out=(qx, sx, h)),
                    lambda wp, N, h, L2, b, y: svdq.linear_w4a4(qx, sx, wp, N, h, L2, b, out=y), 4 * (K // 64))
        sx = torch.empty(((K // 64 + 1) // 2, M, 2, 2), dtype=torch.uint8, device=device)
        return (svdq.pack_weight_mxfp4,
                lambda x, il, rho, l1p, r, h: svdq.quantize_act_mxfp4(x, il, rho, l1p, r, out=(qx, sx, h)),
                lambda wp, N, h, L2, b, y: svdq.linear_mxfp4(qx, sx, wp, N, h, L2, b, out=y), K // 32)

    def measure(fmt):
        """One pass of the hot path per step for the given execution; returns the timing record."""
        w = synth.workload(args.workload, fmt="mxfp4" if fmt == "mxfp4" else "int4")
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
        packer, quant, gemm, scale_bytes = kernels_of(fmt, K, M, x0.device)
        wp = packer(dev(L.qw), dev(L.sw))

        def step(i, ev=None):
            rho = table[i % len(table)]
            if ev:
                ev[0].record()
            quant(xs[i % len(xs)], inv_lambda, rho, l1p, r, h)
            if ev:
                ev[1].record()
            gemm(wp, N, h, L2, bias, ysets[i % len(ysets)])
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
        w = synth.workload(args.workload, fmt="mxfp4" if fmt == "mxfp4" else "int4")
        M = w.M
        xdev = {k: dev(v) for k, v in w.x.items()}
        packer = {"e3m2": svdq.pack_weight_e3m2, "int4": svdq.pack_weight, "mxfp4": svdq.pack_weight_mxfp4}[fmt]
        per_expert = {}
        for ename in w.experts:
            lins = []
            for lin, inp in w.inputs_of.items():
                L = w.layers[f"{ename}/{lin}"]
                inv_lambda = dev(L.inv_lambda)
                rec = dict(L=L, x=xdev[inp], inv_lambda=inv_lambda, L2=dev(L.L2), bias=dev(L.bias),
                           l1p=svdq.pack_lowrank_down(dev(L.L1), inv_lambda),
                           wp=packer(dev(L.qw), dev(L.sw)))
                lins.append(rec)
            per_expert[ename] = lins
        bufs = {}
        for rec in per_expert[w.experts[0]]:
            K, N, r = rec["L"].K, rec["L"].N, rec["L"].r
            if (K, N) not in bufs:
                _, quant, gemm, _ = kernels_of(fmt, K, M, "cuda")
                bufs[(K, N)] = (quant, gemm, torch.empty((M, r), dtype=torch.float32, device="cuda"),
                                torch.empty((M, N), dtype=torch.bfloat16, device="cuda"))

        def step(i, evs=None):
            t = i % w.nsteps
            e = 0 if t < w.switch_step else 1
            step0 = 0 if e == 0 else w.switch_step
            nst = w.switch_step if e == 0 else w.nsteps - w.switch_step
            rho = svdq.alpha_lookup(w.tables[w.experts[e]], t, step0, nst)
            for li, rec in enumerate(per_expert[w.experts[e]]):
                L = rec["L"]
                quant, gemm, h, y = bufs[(L.K, L.N)]
                if evs:
                    evs[li][0].record()
                quant(rec["x"], rec["inv_lambda"], rho, rec["l1p"], L.r, h)
                if evs:
                    evs[li][1].record()
                gemm(rec["wp"], L.N, h, rec["L2"], rec["bias"], y)
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
        sb = (lambda K: K // 32) if fmt == "mxfp4" else (lambda K: 4 * (K // 64))
        bytes_q = sum(M * (2 * rec["L"].K + rec["L"].K // 2 + sb(rec["L"].K) + 4 * rec["L"].r) for rec in per_expert[w.experts[0]])
        return dict(w=w, M=M, ms_step=(t1 - t0) * 1e3 / args.steps, tq=tq, tg=tg, ops=ops, bytes_q=bytes_q, nl=nl)

    def ffn_chain(fmt):
        """Up-projection (workload 3's layer and input) -> GELU -> quantise -> down-projection (workload 4's layer),
        as three kernels and as two (the up-projection's epilogue emits the down-projection's operands)."""
        f = "mxfp4" if fmt == "mxfp4" else "int4"
        wu, wd = synth.workload(2, fmt=f), synth.workload(3, fmt=f)
        Lu, Ld = wu.layers["e0/lin"], wd.layers["e0/lin"]
        M, D, F, r = wu.M, Lu.K, Lu.N, Lu.r
        mk = lambda L, pack: dict(il=dev(L.inv_lambda), L2=dev(L.L2), bias=dev(L.bias), wp=pack(dev(L.qw), dev(L.sw)))
        pack = svdq.pack_weight_mxfp4 if fmt == "mxfp4" else svdq.pack_weight_e3m2
        U, Dn = mk(Lu, pack), mk(Ld, pack)
        U["l1p"] = svdq.pack_lowrank_down(dev(Lu.L1), U["il"])
        Dn["l1p"] = svdq.pack_lowrank_down(dev(Ld.L1), Dn["il"])
        x = dev(wu.x["x"])
        y = torch.empty((M, F), dtype=torch.bfloat16, device="cuda")
        yo = torch.empty((M, D), dtype=torch.bfloat16, device="cuda")
        rho_u, rho_d = wu.tables["e0"][0], wd.tables["e0"][0]
        if fmt == "mxfp4":
            a = svdq.quantize_act_mxfp4(x, U["il"], rho_u, U["l1p"], r)
            up = lambda: svdq.linear_mxfp4(a[0], a[1], U["wp"], F, a[2], U["L2"], U["bias"], out=y)
            up()
            q = svdq.quantize_act_gelu(svdq.FMT_MXFP4, y, Dn["il"], rho_d, Dn["l1p"], r)
            qn = tuple(torch.empty_like(t) for t in q)
            quant = lambda: svdq.quantize_act_gelu(svdq.FMT_MXFP4, y, Dn["il"], rho_d, Dn["l1p"], r, out=q)
            down = lambda b: svdq.linear_mxfp4(b[0], b[1], Dn["wp"], D, b[2], Dn["L2"], Dn["bias"], out=yo)
            upn = lambda: svdq.linear_mxfp4_next(a[0], a[1], U["wp"], F, Dn["il"], rho_d, a[2], U["L2"], U["bias"],
                                                 gelu=True, next_l1_packed=Dn["l1p"], next_r=r, out=qn)
            same = lambda: torch.equal(q[0], qn[0]) and torch.equal(q[1], qn[1])
        else:
            a = svdq.quantize_act_e3m2(x, U["il"], rho_u, U["l1p"], r, want_sx=False)
            up = lambda: svdq.linear_w4a4_e3m2(a[0], U["wp"], F, a[2], U["L2"], U["bias"], out=y)
            up()
            q = svdq.quantize_act_gelu(svdq.FMT_INT4_E3M2, y, Dn["il"], rho_d, Dn["l1p"], r)
            q = (q[0], None, q[2])
            qn = (svdq.ActE3M2(torch.empty_like(q[0].buf), M, F), None, torch.empty_like(q[2]))
            quant = lambda: svdq.quantize_act_gelu(svdq.FMT_INT4_E3M2, y, Dn["il"], rho_d, Dn["l1p"], r, out=q)
            down = lambda b: svdq.linear_w4a4_e3m2(b[0], Dn["wp"], D, b[2], Dn["L2"], Dn["bias"], out=yo)
            upn = lambda: svdq.linear_w4a4_e3m2_next(a[0], U["wp"], F, Dn["il"], rho_d, a[2], U["L2"], U["bias"],
                                                     gelu=True, next_l1_packed=Dn["l1p"], next_r=r, out=qn)
            same = lambda: torch.equal(q[0].buf, qn[0].buf)

        def timed(fn, n=max(4, args.steps // 5)):
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n

        quant(), upn()
        torch.cuda.synchronize()
        rec = {"operands_identical": bool(same()),
               "h_rel_diff": float((q[2] - qn[2]).norm() / q[2].norm()),
               "up_ms": timed(up), "gelu_quantize_ms": timed(quant), "down_ms": timed(lambda: down(q)),
               "up_emitting_ms": timed(upn),
               "unfused_chain_ms": timed(lambda: (up(), quant(), down(q))),
               "fused_chain_ms": timed(lambda: (upn(), down(qn)))}
        rec["fused_over_unfused"] = rec["fused_chain_ms"] / rec["unfused_chain_ms"]
        return rec

    METRIC = "W4A4 SVDQuant linear effective TOPS + % int8-MFMA peak; quantize pass GB/s"
    DTYPE = ("int4 x int4 -> exact integer group sums (codes held as E3M2 fields, FP6 MFMA, binary32 accumulate), "
             "fp32 dequant, bf16 out")

    def rooflines(R, fmt, wname, launches=""):
        """roofline objects of the GEMM and the quantise kernel of one execution."""
        g = R["ops"] / (R["tg"].mean() * 1e-3) / 1e12
        q = R["bytes_q"] / (R["tq"].mean() * 1e-3) / 1e9
        gk, qk, peak, unit = {
            "e3m2": ("svdq_linear_w4a4_e3m2 (gemm_e3m2_kernel)", "svdq_quantize_act_e3m2 (quantize_kernel)",
                     FP6_MFMA_PEAK_TFLOPS, "TFLOP/s"),
            "int4": ("svdq_linear_w4a4 (gemm_kernel)", "svdq_quantize_act (quantize_kernel)", INT8_MFMA_PEAK_TOPS, "TOP/s"),
            "mxfp4": ("svdq_linear_mxfp4 (gemm_mx_kernel)", "svdq_quantize_act_mxfp4 (quantize_mx_kernel)",
                      FP4_MFMA_PEAK_TFLOPS, "TFLOP/s")}[fmt]
        kn = lambda k: k[k.index("(") + 1:-1]
        rg = {"kernel": gk + launches, "bound": "mfma", "achieved": g, "peak": peak, "unit": unit, "frac": g / peak,
              "traffic": measured_traffic(wname, kn(gk)) if wname else None,
              "avg_ms": float(R["tg"].mean()), "min_ms": float(R["tg"].min())}
        if fmt == "e3m2":
            rg["frac_of_int8_peak"] = g / INT8_MFMA_PEAK_TOPS      # the same work priced at the int8 rate
        rq = {"kernel": qk + launches, "bound": "hbm", "achieved": q, "peak": HBM_PEAK_GBS, "unit": "GB/s",
              "frac": q / HBM_PEAK_GBS, "traffic": measured_traffic(wname, kn(qk) + ("_e3m2" if fmt == "e3m2" else "")) if wname else None,
              "algorithmic_bytes": R["bytes_q"], "avg_ms": float(R["tq"].mean()), "min_ms": float(R["tq"].min())}
        return rg, rq

    def variant(R, fmt, what, wname, launches=""):
        rg, rq = rooflines(R, fmt, wname, launches)
        v = {"what": what, "value": R["ops"] / (R["ms_step"] * 1e-3) / 1e12,
             "unit": "TFLOP/s" if fmt == "mxfp4" else "TOPS", "ms_per_step": R["ms_step"],
             "roofline": rg, "roofline_quantize": rq}
        if "bf16_ms" in R:
            v["speedup_vs_bf16_dense"] = R["bf16_ms"] / R["ms_step"]
        return v

    NIBBLE = "same int4 layer on 4-bit storage: nibbles unpacked in registers, int8 matrix cores"
    MXFP4 = "same layer in the MXFP4 format of the paper's Table I on the block-scaled FP4 matrix instruction"

    if args.workload == 4:
        B = measure_block("e3m2")
        rg, rq = rooflines(B, "e3m2", None, ", six launches")
        out = {
            "metric": METRIC, "value": B["ops"] / (B["ms_step"] * 1e-3) / 1e12, "unit": "TOPS",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": B["ms_step"],
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": DTYPE, "data": "synthetic",
            "config": {"workload": f"{B['w'].name}: M={B['M']}, six linears (q, k, v, o 5120x5120; ffn_up 5120x13824; "
                                   f"ffn_down 13824x5120) r=32, two experts over a 40-step schedule, ratio per timestep bin",
                       "step": f"{B['nl']} x (svdq_quantize_act_e3m2 + svdq_linear_w4a4_e3m2) = one DiT block-step"},
            "roofline": rg, "roofline_quantize": rq,
        }
        del B
        out["int4_nibble_variant"] = variant(measure_block("int4"), "int4", NIBBLE, None, ", six launches")
        if not args.skip_mxfp4:
            out["mxfp4_variant"] = variant(measure_block("mxfp4"), "mxfp4", MXFP4, None, ", six launches")
        print(json.dumps(out))
        return

    R = measure("e3m2")
    w, L, table, M, K, N, r = R["w"], R["L"], R["table"], R["M"], R["K"], R["N"], R["r"]
    rg, rq = rooflines(R, "e3m2", w.name)
    out = {
        "metric": METRIC, "value": R["ops"] / (R["ms_step"] * 1e-3) / 1e12, "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": R["ms_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": f"{w.name}: M={M} K={K} N={N} r={r} group=64, rho per timestep bin {table}",
                   "step": "svdq_quantize_act_e3m2 + svdq_linear_w4a4_e3m2", "input_sets": R["nx"]},
        "roofline": rg, "roofline_quantize": rq,
        "context": {"bf16_dense_matmul_ms": R["bf16_ms"], "speedup_vs_bf16_dense": R["bf16_ms"] / R["ms_step"],
                    "note": "vendor-library bf16 GEMM of the same shape on the same GPU (the paper's BF16 baseline)"},
    }
    del R
    out["int4_nibble_variant"] = variant(measure("int4"), "int4", NIBBLE, w.name)
    if not args.skip_mxfp4:
        out["mxfp4_variant"] = variant(measure("mxfp4"), "mxfp4", MXFP4, w.name)
    if args.cpu_rows > 0:
        out["cpu_baseline"] = cpu_baseline(w, L, args.cpu_rows)
    if args.ffn_chain:
        del w, L
        out["ffn_chain"] = {"workload": "c3_ffn_up -> GELU -> c4_ffn_down: M=32760, 5120 -> 13824 -> 5120, r=32",
                            "int4_e3m2": ffn_chain("e3m2")}
        if not args.skip_mxfp4:
            out["ffn_chain"]["mxfp4"] = ffn_chain("mxfp4")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
