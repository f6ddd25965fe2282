"""Host-side checks of the C-ABI library: it loads, exports what include/svdq.h declares,
validates arguments before touching a GPU, and its host helper matches the oracle."""
import ctypes
import os
import re

import numpy as np

import paper_2605_27003_amd as svdq
from paper_2605_27003_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "svdq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(svdq_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = svdq.load_library()
    names = declared_functions()
    assert len(names) >= 11
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(binding.EXPORTS)


def test_sizes_and_version():
    assert svdq.version() >= 1
    assert svdq.packed_l1_bytes(5120) == 5120 * 128
    assert svdq.packed_l1_bytes(100) == 0
    assert svdq.packed_weight_bytes(5120, 5120) >= 5120 * 2560
    assert svdq.packed_weight_bytes(100, 5120) == 0


def test_argument_errors_before_any_launch():
    lib = svdq.load_library()
    a = ctypes.c_void_p(256)                     # never dereferenced: checks fail first
    z = ctypes.c_void_p(0)
    INV, SHAPE = -1, -2
    q = lib.svdq_quantize_act
    assert q(z, 512, a, 0.9, z, 4, 512, 0, a, a, z, z) == INV                 # NULL x
    assert q(a, 512, a, 0.0, z, 4, 512, 0, a, a, z, z) == INV                 # rho = 0
    assert q(a, 512, a, 1.5, z, 4, 512, 0, a, a, z, z) == INV                 # rho > 1
    assert q(a, 512, a, float("nan"), z, 4, 512, 0, a, a, z, z) == INV
    assert q(a, 512, a, 0.9, z, -1, 512, 0, a, a, z, z) == INV                # M < 0
    assert q(a, 512, a, 0.9, z, 4, 512, 16, a, a, z, z) == INV                # r without packed L1
    assert q(a, 512, a, 0.9, a, 4, 512, 16, a, a, z, z) == INV                # packed L1 without h
    assert q(a, 512, a, 0.9, z, 4, 500, 0, a, a, z, z) == SHAPE               # K % 64
    assert q(a, 256, a, 0.9, z, 4, 512, 0, a, a, z, z) == SHAPE               # ldx < K
    assert q(a, 512, a, 0.9, a, 4, 512, 8, a, a, a, z) == SHAPE               # rank 8
    assert q(ctypes.c_void_p(260), 512, a, 0.9, z, 4, 512, 0, a, a, z, z) == SHAPE   # misaligned
    assert q(a, 512, a, 0.9, z, 0, 512, 0, a, a, z, z) == 0                   # M == 0 no-op
    g = lib.svdq_linear_w4a4
    assert g(z, a, a, z, z, z, 4, 512, 512, 0, a, 512, 0, z) == INV
    assert g(a, a, a, a, z, z, 4, 512, 512, 16, a, 512, 0, z) == INV          # h without L2
    assert g(a, a, a, z, z, z, 4, 512, 512, 0, a, 512, 7, z) == INV           # bad out dtype
    assert g(a, a, a, z, z, z, 4, 500, 512, 0, a, 512, 0, z) == SHAPE         # N % 128
    assert g(a, a, a, z, z, z, 4, 512, 512, 0, a, 256, 0, z) == SHAPE         # ldy < N
    assert g(a, a, a, z, z, z, 0, 512, 512, 0, a, 512, 0, z) == 0
    assert lib.svdq_pack_weight(z, a, 512, 512, a, z) == INV
    assert lib.svdq_pack_weight(a, a, 512, 100, a, z) == SHAPE
    assert lib.svdq_pack_lowrank_down(a, z, 512, 16, a, z) == INV
    assert lib.svdq_pack_lowrank_down(a, a, 512, 24, a, z) == SHAPE
    assert lib.svdq_lowrank(2, a, 512, a, a, 4, 512, 512, 16, a, a, 512, z) == INV
    assert lib.svdq_debug_group_acc(a, a, 4, 512, 512, 2, 8, a, z) == INV     # rows beyond M
    assert lib.svdq_debug_scale_chain(a, 1.5, 4, a, a, z) == INV
    assert lib.svdq_debug_scale_chain(a, 0.5, 0, a, a, z) == 0
    # MXFP4 variant: same conventions
    qm = lib.svdq_quantize_act_mxfp4
    assert qm(z, 512, a, 0.9, z, 4, 512, 0, a, a, z, z) == INV                # NULL x
    assert qm(a, 512, a, 0.0, z, 4, 512, 0, a, a, z, z) == INV                # rho = 0
    assert qm(a, 512, a, 0.9, z, 4, 512, 16, a, a, z, z) == INV               # r without packed L1
    assert qm(a, 512, a, 0.9, z, 4, 480, 0, a, a, z, z) == SHAPE              # K % 64
    assert qm(a, 512, a, 0.9, z, 0, 512, 0, a, a, z, z) == 0                  # M == 0 no-op
    gm = lib.svdq_linear_mxfp4
    assert gm(z, a, a, z, z, z, 4, 512, 512, 0, a, 512, 0, z) == INV
    assert gm(a, a, a, a, z, z, 4, 512, 512, 16, a, 512, 0, z) == INV         # h without L2
    assert gm(a, a, a, z, z, z, 4, 500, 512, 0, a, 512, 0, z) == SHAPE        # N % 128
    assert gm(a, a, a, z, z, z, 0, 512, 512, 0, a, 512, 0, z) == 0
    gmn = lib.svdq_linear_mxfp4_next
    assert gmn(a, a, a, z, z, z, 4, 512, 512, 0, 1, a, 0.9, z, 0, a, z, z, z) == INV      # no scale output
    assert gmn(a, a, a, z, z, z, 4, 512, 512, 0, 1, a, 0.9, a, 16, a, a, z, z) == INV     # next L1 without next h
    assert gmn(a, a, a, z, z, z, 4, 500, 512, 0, 1, a, 0.9, z, 0, a, a, z, z) == SHAPE
    assert gmn(a, a, a, z, z, z, 0, 512, 512, 0, 1, a, 0.9, z, 0, a, a, z, z) == 0
    assert lib.svdq_pack_weight_mxfp4(z, a, 512, 512, a, z) == INV
    assert lib.svdq_pack_weight_mxfp4(a, a, 512, 100, a, z) == SHAPE
    assert svdq.packed_weight_mxfp4_bytes(5120, 5120) >= 5120 * 2560 and svdq.packed_weight_mxfp4_bytes(100, 5120) == 0
    # E3M2-container execution: same conventions
    q6 = lib.svdq_quantize_act_e3m2
    assert q6(z, 512, a, 0.9, z, 4, 512, 0, a, a, z, z) == INV                # NULL x
    assert q6(a, 512, a, 0.9, z, 4, 512, 0, z, a, z, z) == INV                # NULL operand buffer
    assert q6(a, 512, a, 1.5, z, 4, 512, 0, a, z, z, z) == INV                # rho > 1
    assert q6(a, 512, a, 0.9, z, 4, 512, 16, a, z, z, z) == INV               # r without packed L1
    assert q6(a, 512, a, 0.9, z, 4, 480, 0, a, z, z, z) == SHAPE              # K % 64
    assert q6(a, 512, a, 0.9, z, 0, 512, 0, a, z, z, z) == 0                  # M == 0 no-op, sx optional
    g6 = lib.svdq_linear_w4a4_e3m2
    assert g6(z, a, z, z, z, 4, 512, 512, 0, a, 512, 0, z) == INV
    assert g6(a, a, a, z, z, 4, 512, 512, 16, a, 512, 0, z) == INV            # h without L2
    assert g6(a, a, z, z, z, 4, 500, 512, 0, a, 512, 0, z) == SHAPE           # N % 128
    assert g6(a, a, z, z, z, 0, 512, 512, 0, a, 512, 0, z) == 0
    gn = lib.svdq_linear_w4a4_e3m2_next                                         # two layers fused across their boundary
    assert gn(a, a, z, z, z, 4, 512, 512, 0, 1, z, 0.9, z, 0, a, z, z, z) == INV      # no smoothing vector of the next layer
    assert gn(a, a, z, z, z, 4, 512, 512, 0, 1, a, 0.9, z, 0, z, z, z, z) == INV      # no output buffer
    assert gn(a, a, z, z, z, 4, 512, 512, 0, 1, a, 1.5, z, 0, a, z, z, z) == INV      # next rho > 1
    assert gn(a, a, z, z, z, 4, 512, 512, 0, 1, a, 0.9, a, 16, a, z, z, z) == INV     # next L1 without next h
    assert gn(a, a, z, z, z, 4, 512, 512, 0, 1, a, 0.9, z, 16, a, z, z, z) == INV     # next rank without next L1
    assert gn(a, a, z, z, z, 4, 500, 512, 0, 1, a, 0.9, z, 0, a, z, z, z) == SHAPE
    assert gn(a, a, z, z, z, 4, 512, 512, 0, 1, a, 0.9, a, 8, a, z, a, z) == SHAPE    # next rank 8
    assert gn(a, a, z, z, z, 0, 512, 512, 0, 1, a, 0.9, z, 0, a, z, z, z) == 0
    assert lib.svdq_pack_weight_e3m2(z, a, 512, 512, a, z) == INV
    assert lib.svdq_pack_weight_e3m2(a, a, 512, 100, a, z) == SHAPE
    assert lib.svdq_unpack_act_e3m2(a, 4, 100, a, z) == SHAPE
    assert lib.svdq_unpack_act_e3m2(a, 0, 128, a, z) == 0
    assert lib.svdq_debug_group_acc_e3m2(a, a, 4, 512, 512, 2, 8, a, z) == INV   # rows beyond M
    assert svdq.packed_weight_e3m2_bytes(5120, 5120) == 5120 * 80 * 56 and svdq.packed_weight_e3m2_bytes(100, 5120) == 0
    assert svdq.act_e3m2_bytes(5, 128) == 2 * 8 * 56 and svdq.act_e3m2_bytes(5, 100) == 0
    # activation fused into kernel (a): the format selector, then that format's checks
    qg = lib.svdq_quantize_act_gelu
    assert qg(9, a, 512, a, 0.9, z, 4, 512, 0, a, a, z, z) == INV              # unknown format
    for fmt in (0, 1, 2):
        assert qg(fmt, z, 512, a, 0.9, z, 4, 512, 0, a, a, z, z) == INV        # NULL x
        assert qg(fmt, a, 512, a, 0.9, z, 4, 480, 0, a, a, z, z) == SHAPE      # K % 64
        assert qg(fmt, a, 512, a, 0.9, z, 0, 512, 0, a, a, z, z) == 0          # M == 0 no-op
    assert lib.svdq_debug_gelu(z, 4, a, z) == INV and lib.svdq_debug_gelu(a, 0, a, z) == 0
    # GPTQ calibration
    assert lib.svdq_gptq_workspace_bytes(128, 100) == 0 and lib.svdq_gptq_workspace_bytes(128, 128) >= 128 * 128 * 17
    assert lib.svdq_gptq_hessian(z, 128, a, 4, 128, a, z) == INV
    assert lib.svdq_gptq_hessian(a, 64, a, 4, 128, a, z) == SHAPE               # ldx < K
    assert lib.svdq_gptq_hessian(a, 128, a, 0, 128, a, z) == 0
    assert lib.svdq_gptq_quantize(a, a, -1.0, 128, 128, a, a, a, z) == INV      # negative damping
    assert lib.svdq_gptq_quantize(a, a, 0.01, 128, 100, a, a, a, z) == SHAPE
    assert lib.svdq_gptq_quantize(a, z, 0.01, 128, 128, a, a, a, z) == INV
    # clipping-ratio search: reduction, accumulation over a bin's steps, arg-min over the candidates
    for f in (lib.svdq_sq_error, lib.svdq_sq_error_add):
        assert f(z, 64, a, 64, 4, 64, a, a, z) == INV
        assert f(a, 64, a, 64, 4, 64, z, a, z) == INV                            # no workspace
        assert f(a, 64, a, 64, 4, 60, a, a, z) == SHAPE                          # N % 8
        assert f(a, 32, a, 64, 4, 64, a, a, z) == SHAPE                          # ld_ref < N
    assert lib.svdq_argmin_rows(z, 4, 5, a, z) == INV and lib.svdq_argmin_rows(a, 4, 0, a, z) == INV
    assert lib.svdq_argmin_rows(a, 0, 5, a, z) == 0
    # the same reduction without a workspace (static device scratch): same checks plus its size limit
    fs = lib.svdq_sq_error_static
    assert fs(z, 64, a, 64, 4, 64, a, z) == INV and fs(a, 64, a, 64, 4, 64, z, z) == INV
    assert fs(a, 64, a, 64, 4, 60, a, z) == SHAPE and fs(a, 64, a, 32, 4, 64, a, z) == SHAPE
    assert fs(a, 1 << 20, a, 1 << 20, (1 << 16) + 1, 1 << 20, a, z) == SHAPE     # more than 2^36 elements
    # token counts beyond what the kernels' 32-bit per-lane offsets cover
    big = (1 << 26) + 1
    assert q(a, 512, a, 0.9, z, big, 512, 0, a, a, z, z) == SHAPE
    assert g(a, a, a, z, z, z, big, 512, 512, 0, a, 512, 0, z) == SHAPE
    assert q6(a, 512, a, 0.9, z, big, 512, 0, a, z, z, z) == SHAPE
    assert g6(a, a, z, z, z, big, 512, 512, 0, a, 512, 0, z) == SHAPE
    assert qm(a, 512, a, 0.9, z, big, 512, 0, a, a, z, z) == SHAPE
    assert gm(a, a, a, z, z, z, big, 512, 512, 0, a, 512, 0, z) == SHAPE
    assert lib.svdq_status_string(-2) == b"unsupported shape"


def test_alpha_lookup_matches_oracle(oracle):
    table = [0.9, 0.8, 0.8, 0.9, 0.7, 0.8, 0.6, 1.0]
    for nbins in (1, 4, 8):
        for step0, n in ((0, 20), (20, 20), (0, 40), (5, 3)):
            for step in range(step0 - 2, step0 + n + 2):
                a = svdq.alpha_lookup(table[:nbins], step, step0, n)
                b = oracle.alpha_lookup(table[:nbins], step, step0, n)
                assert (np.isnan(a) and np.isnan(b)) or a == b
