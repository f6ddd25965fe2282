"""GPU-vs-oracle parity at the benchmark's full sizes, in the launch configuration bench.py times.

Rows are independent in this path, so a row sample checked against the oracle
is exact for those rows.  Both executions of the int4 layer are covered: 4-bit
storage on the int8 matrix cores, and E3M2 fields on the FP6 matrix cores.  Per configuration: int4 codes and scales over the
WHOLE buffers (bit-exact), h over the whole buffer, int32 group accumulators of
the first rows and of the ragged last tile (bit-exact), and the bf16 / f32
output on a seeded row sample (first 64, last 64, random rows).
"""
import os
import time

import numpy as np
import pytest
import torch

from workloads import synth
from tests.helpers import DeviceLayer, check_y, dev, host_bits, rel_fro

pytestmark = pytest.mark.gpu
T0 = time.time()


def progress(msg):
    """One line per finished step, also appended to the file SVDQ_PROGRESS_LOG names when it is set (pytest holds
    back stdout; a long step must not look hung)."""
    line = f"[{time.time() - T0:7.1f}s] {msg}"
    print(line, flush=True)
    log = os.environ.get("SVDQ_PROGRESS_LOG")
    if log:
        with open(log, "a") as f:
            f.write(line + "\n")


@pytest.fixture(scope="module")
def svdq():
    import paper_2605_27003_amd as m
    m.load_library(build_if_missing=False)
    return m


def check_layer(svdq, oracle, name, x_bits, x_dev, L, DL, rho, n_sample, whole, acc_rows=64, seed=1):
    """One (input, layer, rho): quantise + GEMM on the full M on the GPU, oracle on what it can afford."""
    M = x_bits.shape[0]
    qx, sx, h = svdq.quantize_act(x_dev, DL.inv_lambda, rho, DL.l1p, L.r)
    y16 = svdq.linear_w4a4(qx, sx, DL.wp, L.N, h, DL.L2, DL.bias)
    torch.cuda.synchronize()
    S = synth.sample_rows(M, n_sample - 128, seed)
    St = torch.from_numpy(S).cuda()
    xs = np.ascontiguousarray(x_bits[S])
    oq, os_ = oracle.quantize_act(xs, L.inv_lambda, rho)
    # the library's codes/scales are group-major [K/64, M, ...]; gather the sampled rows and permute
    gq = qx[:, St].permute(1, 0, 2).reshape(len(S), -1).cpu().numpy()
    gs = sx[:, St].t().contiguous().cpu().numpy()
    assert np.array_equal(gq, oq), f"{name}: codes (row sample)"
    assert np.array_equal(gs.view(np.uint32), os_.view(np.uint32)), f"{name}: scales (row sample)"
    oh = oracle.lowrank_down(xs, L.inv_lambda, L.L1)
    assert rel_fro(h[St].cpu().numpy(), oh) <= 3e-5, f"{name}: h (row sample)"
    progress(f"{name} rho={rho}: codes/scales/h ok on {len(S)} rows")
    if whole:
        fq, fs = oracle.quantize_act(x_bits, L.inv_lambda, rho)
        wq, ws = svdq.to_token_major(qx, sx)
        assert np.array_equal(ws.cpu().numpy().view(np.uint32), fs.view(np.uint32)), f"{name}: scales (whole buffer)"
        assert np.array_equal(wq.cpu().numpy(), fq), f"{name}: codes (whole buffer)"
        del fq, fs, wq, ws
        progress(f"{name} rho={rho}: whole-buffer codes/scales ok ({M}x{L.K})")
        if whole > 1:
            fh = oracle.lowrank_down(x_bits, L.inv_lambda, L.L1)
            assert rel_fro(h.cpu().numpy(), fh) <= 3e-5, f"{name}: h (whole buffer)"
            del fh
        for m0 in (0, M - acc_rows):
            acc = svdq.debug_group_acc(qx, DL.wp, L.N, m0, acc_rows).cpu().numpy()
            want = oracle.group_acc(qx[:, m0:m0 + acc_rows].permute(1, 0, 2).reshape(acc_rows, -1).cpu().numpy(), L.qw)
            assert np.array_equal(acc, want), f"{name}: group accumulators rows {m0}.."
            del acc, want
        progress(f"{name}: group accumulators (first rows, ragged last tile) ok")
    y32 = svdq.linear_w4a4(qx, sx, DL.wp, L.N, h, DL.L2, DL.bias, out_dtype=torch.float32)
    torch.cuda.synchronize()
    orc = oracle.linear(oq, os_, L.qw, L.sw, oh, L.L2, L.bias)
    stats = check_y(host_bits(y16[St]), y32[St].cpu().numpy(), orc, name)
    del y32, y16
    progress(f"{name} rho={rho}: y ok on {len(S)} rows {stats}")

    # The same layer with the codes held as E3M2 fields on the FP6 matrix cores (the execution bench.py times).
    # Its operand buffer must hold exactly the codes checked above (whole buffer, compared on the device after the
    # library's conversion back to nibbles; the sampled rows also decoded on the host straight from the documented
    # layout), its group sums must be the oracle's, and its y meets the same bar.
    act, _, h6 = svdq.quantize_act_e3m2(x_dev, DL.inv_lambda, rho, DL.l1p, L.r, want_sx=False)
    assert torch.equal(svdq.unpack_act_e3m2(act), qx), f"{name}: E3M2 codes (whole buffer)"
    assert torch.equal(h6, h), f"{name}: h of the E3M2 quantise pass"
    Mp, ng = (M + 3) // 4 * 4, L.K // 64
    blk = act.buf.view(ng, Mp * 56)
    rows = torch.cat([blk[:, : Mp * 32].reshape(ng, Mp, 32)[:, St].reshape(ng, len(S), 2, 16),
                      blk[:, Mp * 32: Mp * 48].reshape(ng, 2, Mp, 8)[:, :, St].permute(0, 2, 1, 3)], dim=-1).cpu().numpy()
    bits = np.unpackbits(rows, axis=-1, bitorder="little").reshape(ng, len(S), 2, 32, 6)
    f = (bits * (1 << np.arange(6))).sum(-1)
    val = np.where((f >> 2) & 7, (4 + (f & 3)) * 2.0 ** (((f >> 2) & 7) - 5.0), (f & 3) / 16.0) * np.where(f >> 5, -1.0, 1.0)
    assert np.array_equal(val.transpose(1, 0, 2, 3).reshape(len(S), L.K), synth.unpack_int4(oq)), f"{name}: E3M2 fields (row sample)"
    del rows, bits, f, val
    # the scale-piece plane: per (group, token) the pair {p, p}, p = hi | lo << 16 with hi = bf16(s), lo = bf16(s - hi)
    # of the oracle's binary32 scale s (round to nearest even, torch's cast): sampled rows against the oracle, and
    # the whole plane against the same split of the scales that were compared with the oracle above
    def pieces(s32):                                           # torch tensor of binary32 scales -> uint32 p (as int64)
        hi = s32.to(torch.bfloat16)
        lo = (s32 - hi.float()).to(torch.bfloat16)
        return (hi.view(torch.int16).to(torch.int64) & 0xFFFF) | ((lo.view(torch.int16).to(torch.int64) & 0xFFFF) << 16)
    plane = blk[:, Mp * 48:].reshape(ng, Mp, 8)[:, :M].contiguous().view(torch.int32).to(torch.int64) & 0xFFFFFFFF
    assert torch.equal(plane[..., 0], plane[..., 1]), f"{name}: scale pieces are stored twice"
    want_s = pieces(torch.from_numpy(os_).t().contiguous())                     # [ng, |S|] from the ORACLE's scales
    assert torch.equal(plane[:, St, 0].cpu(), want_s), f"{name}: E3M2 scale pieces (row sample, oracle scales)"
    assert torch.equal(plane[..., 0], pieces(sx)), f"{name}: E3M2 scale pieces (whole plane)"
    del plane, want_s
    if whole:
        for m0 in (0, M - acc_rows):
            acc = svdq.debug_group_acc_e3m2(act, DL.wp6, L.N, m0, acc_rows).cpu().numpy()
            want = oracle.group_acc(qx[:, m0:m0 + acc_rows].permute(1, 0, 2).reshape(acc_rows, -1).cpu().numpy(), L.qw)
            assert np.array_equal(acc, want), f"{name}: E3M2 group sums rows {m0}.."
            del acc, want
    y16 = svdq.linear_w4a4_e3m2(act, DL.wp6, L.N, h6, DL.L2, DL.bias)
    y32 = svdq.linear_w4a4_e3m2(act, DL.wp6, L.N, h6, DL.L2, DL.bias, out_dtype=torch.float32)
    torch.cuda.synchronize()
    stats = check_y(host_bits(y16[St]), y32[St].cpu().numpy(), orc, name + " e3m2")
    del y32, y16, act
    progress(f"{name} rho={rho}: E3M2 execution ok (codes whole buffer, y on {len(S)} rows) {stats}")


@pytest.mark.parametrize("idx", [1, 2, 3])
def test_single_linear_configs(svdq, oracle, idx):
    w = synth.workload(idx)
    progress(f"{w.name}: inputs generated (M={w.M})")
    L, x = w.layers["e0/lin"], w.x["x"]
    DL = DeviceLayer(L)
    xd = dev(x)
    table = w.tables["e0"]
    seen = []
    for b, rho in enumerate(table):
        if rho in seen:
            continue
        check_layer(svdq, oracle, f"{w.name}/bin{b}", x, xd, L, DL, rho,
                    n_sample=2048 if not seen else 512, whole=0 if seen else 2, seed=idx * 10 + b)
        seen.append(rho)


@pytest.fixture(scope="module")
def block720p():
    w = synth.workload(4)
    progress(f"{w.name}: inputs generated (M={w.M}, {len(w.layers)} layers)")
    return w


@pytest.mark.parametrize("expert", ["high_noise", "low_noise"])
def test_block_720p_schedule(svdq, oracle, block720p, expert):
    """Both experts over the 40-step schedule (switch at step 20): first and last step of each expert
    and one step in every other timestep bin; all six linears; x changes with the step (row rotation)."""
    w = block720p
    step0 = 0 if expert == "high_noise" else w.switch_step
    nsteps = w.switch_step if expert == "high_noise" else w.nsteps - w.switch_step
    table = w.tables[expert]
    steps, bins = [], set()
    for s in [step0, step0 + nsteps - 1] + list(range(step0, step0 + nsteps)):
        b = ((s - step0) * len(table)) // nsteps
        if s in (step0, step0 + nsteps - 1) or b not in bins:
            if s not in steps:
                steps.append(s)
            bins.add(b)
    assert bins == set(range(len(table)))
    xdev = {k: dev(v) for k, v in w.x.items()}
    layers = {lin: DeviceLayer(w.layers[f"{expert}/{lin}"]) for lin in w.inputs_of}
    for si, step in enumerate(steps):
        rho = svdq.alpha_lookup(table, step, step0, nsteps)
        assert rho == oracle.alpha_lookup(table, step, step0, nsteps)
        shift = (step * 997) % w.M
        for lin, inp in w.inputs_of.items():
            DL = layers[lin]
            xb = np.roll(w.x[inp], shift, axis=0) if si == 0 and lin in ("q", "ffn_down") else None
            xd = torch.roll(xdev[inp], shift, dims=0)
            if xb is None:                                   # only the sampled rows are needed on the host
                class _Rows:                                 # lazy rolled view: x_step[i] = x[(i - shift) % M]
                    shape = w.x[inp].shape
                    def __getitem__(self, S, _x=w.x[inp], _s=shift, _M=w.M):
                        return _x[(np.asarray(S) - _s) % _M]
                xb = _Rows()
            check_layer(svdq, oracle, f"{w.name}/{expert}/step{step}/{lin}", xb, xd, DL.L, DL, rho,
                        n_sample=256, whole=int(si == 0 and lin in ("q", "ffn_down")), seed=step)
            del xd
    # one step per expert on FRESH activations (new values of the same distribution, seeded by the step) for the
    # down-projection, the layer whose post-GELU input the paper singles out: 2048 sampled rows
    step = steps[1]
    rho = svdq.alpha_lookup(table, step, step0, nsteps)
    xb, _ = synth.block_input("x_down", w.M, step=step)
    progress(f"{w.name}/{expert}: fresh x_down for step {step} generated")
    check_layer(svdq, oracle, f"{w.name}/{expert}/step{step}/ffn_down/fresh-x", xb, dev(xb), layers["ffn_down"].L,
                layers["ffn_down"], rho, n_sample=2048, whole=0, seed=1000 + step)


@pytest.mark.parametrize("fmt", ["int4", "mxfp4"])
def test_ffn_chain_emitting_epilogue_fullsize(svdq, oracle, fmt):
    """Up-projection (C3) -> GELU -> quantise for the down-projection (C4) at M = 32760, with the GEMM epilogue that
    emits the operands: whole buffers byte-identical to the un-fused sequence; on a row sample (rows are independent
    along the whole chain) bit-exact against the oracle's chain wherever the two sides' bf16 activations agree."""
    from tests.helpers import unpack_act_e3m2_np
    wu, wd = synth.workload(2, fmt=fmt), synth.workload(3, fmt=fmt)
    Lu, Ld = wu.layers["e0/lin"], wd.layers["e0/lin"]
    M, F, r = wu.M, Lu.N, Lu.r
    progress(f"ffn chain {fmt}: inputs generated (M={M})")
    x = wu.x["x"]
    ilu, ild = dev(Lu.inv_lambda), dev(Ld.inv_lambda)
    l1u, l1d = svdq.pack_lowrank_down(dev(Lu.L1), ilu), svdq.pack_lowrank_down(dev(Ld.L1), ild)
    L2u, bu = dev(Lu.L2), dev(Lu.bias)
    rho_u, rho_d = wu.tables["e0"][0], wd.tables["e0"][0]
    S = synth.sample_rows(M, 256, 5)
    St = torch.from_numpy(S).cuda()
    xs = np.ascontiguousarray(x[S])
    if fmt == "mxfp4":
        wp = svdq.pack_weight_mxfp4(dev(Lu.qw), dev(Lu.sw))
        a = svdq.quantize_act_mxfp4(dev(x), ilu, rho_u, l1u, r)
        y = svdq.linear_mxfp4(a[0], a[1], wp, F, a[2], L2u, bu)
        ref = svdq.quantize_act_gelu(svdq.FMT_MXFP4, y, ild, rho_d, l1d, r)
        got = svdq.linear_mxfp4_next(a[0], a[1], wp, F, ild, rho_d, a[2], L2u, bu, gelu=True, next_l1_packed=l1d, next_r=r)
        torch.cuda.synchronize()
        assert torch.equal(got[0], ref[0]) and torch.equal(got[1], ref[1])
        oq, os_ = oracle.quantize_act_mxfp4(xs, Lu.inv_lambda, rho_u)
        orc = oracle.linear_mxfp4(oq, os_, Lu.qw, Lu.sw, oracle.lowrank_down(xs, Lu.inv_lambda, Lu.L1), Lu.L2, Lu.bias,
                                  want=("ybf16",))
        xg = oracle.gelu_tanh_bf16(orc["ybf16"])
        oq2, os2 = oracle.quantize_act_mxfp4(xg, Ld.inv_lambda, rho_d)
        gq, gs = svdq.mx_to_token_major(got[0][:, St].contiguous(), got[1][:, St].contiguous(), F)
        gq, gs, blk = gq.cpu().numpy(), gs.cpu().numpy(), 32
        codes_g, codes_o = gq.reshape(len(S), -1, blk // 2), oq2.reshape(len(S), -1, blk // 2)
    else:
        wp = svdq.pack_weight_e3m2(dev(Lu.qw), dev(Lu.sw))
        a = svdq.quantize_act_e3m2(dev(x), ilu, rho_u, l1u, r, want_sx=False)
        y = svdq.linear_w4a4_e3m2(a[0], wp, F, a[2], L2u, bu)
        ref = svdq.quantize_act_gelu(svdq.FMT_INT4_E3M2, y, ild, rho_d, l1d, r)
        got = svdq.linear_w4a4_e3m2_next(a[0], wp, F, ild, rho_d, a[2], L2u, bu, gelu=True, next_l1_packed=l1d, next_r=r)
        torch.cuda.synchronize()
        # rows M..Mp-1 of the operand buffer are padding that neither call writes; M is a multiple of 4 here
        assert M % 4 == 0 and torch.equal(got[0].buf, ref[0].buf) and torch.equal(got[1], ref[1])
        oq, os_ = oracle.quantize_act(xs, Lu.inv_lambda, rho_u)
        orc = oracle.linear(oq, os_, Lu.qw, Lu.sw, oracle.lowrank_down(xs, Lu.inv_lambda, Lu.L1), Lu.L2, Lu.bias,
                            want=("ybf16",))
        xg = oracle.gelu_tanh_bf16(orc["ybf16"])
        oq2, os2 = oracle.quantize_act(xg, Ld.inv_lambda, rho_d)
        gs = got[1][:, St].t().contiguous().cpu().numpy()
        qn = svdq.unpack_act_e3m2(got[0])                                       # [F/64, M, 32] nibbles
        gq, blk = qn[:, St].permute(1, 0, 2).reshape(len(S), -1).cpu().numpy(), 64
        codes_g, codes_o = gq.reshape(len(S), -1, blk // 2), oq2.reshape(len(S), -1, blk // 2)
    hrel = float((got[2].double() - ref[2].double()).norm() / ref[2].double().norm())
    assert hrel <= 2e-6, hrel
    progress(f"ffn chain {fmt}: operands byte-identical to the un-fused sequence on the whole buffers, h' rel diff {hrel:.2e}")
    same = (host_bits(y[St]) == orc["ybf16"]).reshape(len(S), F // blk, blk).all(axis=2)
    assert same.mean() > 0.03, same.mean()
    sg, so = (gs, os2) if fmt == "mxfp4" else (gs.view(np.uint32), os2.view(np.uint32))
    assert np.array_equal(sg[same], so[same]) and np.array_equal(codes_g[same], codes_o[same])
    oh2 = oracle.lowrank_down(xg, Ld.inv_lambda, Ld.L1)
    hd = rel_fro(got[2][St].cpu().numpy(), oh2)
    assert hd <= 3e-3, hd
    progress(f"ffn chain {fmt}: oracle chain bit-exact on {same.mean() * 100:.1f} % of the sampled (token, block) pairs "
             f"(those whose activations agree), h' rel {hd:.1e}")
