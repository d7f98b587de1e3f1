"""CPU-only checks of the boundary: the library loads, exports every symbol the header declares, its host-side
logic (parameter table, schedules, workspace sizes, argument validation before any HIP call) is right."""
import ctypes as C
import json
import math
import os
import re

import numpy as np
import pytest

from oracle import ops as orc
from oracle import resnet50
from paper_1711_04325_amd import binding as rn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    txt = open(os.path.join(ROOT, "include", "rn50.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\(", " ".join(l for l in txt.splitlines() if not l.startswith("#")))))


def test_every_declared_symbol_is_exported_and_bound():
    names = _declared()
    assert len(names) >= 30
    raw = C.CDLL(rn.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), n
    assert set(names) == set(rn.EXPORTS)


def test_param_table_matches_the_oracles_architecture():
    tab = rn.rn50_param_table()
    ref = resnet50.param_table()
    assert rn.rn50_param_count() == 25_557_032 == resnet50.param_count()
    assert len(tab) == len(ref) == 161
    off = 0
    for (name, o, cnt, dims, kind), (rname, shape, rkind) in zip(tab, ref):
        assert name == rname and rn.KIND_NAMES[kind] == rkind and o == off and cnt == int(np.prod(shape))
        if rkind == "conv_w":
            k, c, r, s = shape
            assert dims == (k, r, s, c)   # device filters are KRSC
        assert o % 64 == 0
        off += cnt


def test_schedules_match_oracle_and_paper(golden_dir):
    gold = json.load(open(os.path.join(golden_dir, "paper_constants.json")))
    for e in np.linspace(0, 90, 361):
        assert abs(rn.rn50_alpha_sgd(e) - orc.alpha_sgd(e)) < 1e-15
        assert abs(rn.rn50_lr_slow_start(e) - orc.lr_slow_start(e)) < 1e-12
    assert rn.rn50_alpha_sgd(gold["beta_center"]) == 0.5 and rn.rn50_alpha_sgd(12.5) == 1.0
    assert abs(rn.rn50_lr_base(1024, 32) - gold["eta_base"]) < 1e-12
    assert abs(rn.rn50_alpha_rmsprop(0.25, 3e-4, 6.4) - orc.alpha_rmsprop(0.25, 3e-4, 6.4)) < 1e-18


def test_rejected_transitions_match_oracle():
    """Appendix A.1's alternative transition functions against the oracle's, and through the per-iteration scalars."""
    for kind in (0, 1, 2, 3):
        for e in np.linspace(0, 30, 241):
            assert abs(rn.rn50_alpha_sgd_transition(e, kind) - orc.alpha_sgd_transition(e, kind)) < 1e-15
        assert abs(rn.rn50_alpha_sgd_transition(4.5, kind, 4.0, 2.0) - orc.alpha_sgd_transition(4.5, kind, 4.0, 2.0)) < 1e-15
    assert math.isnan(rn.rn50_alpha_sgd_transition(1.0, 9))
    for kind in (0, 1, 2, 3):
        for epoch in (0.0, 8.0, 10.0, 11.0, 45.0):
            hp = rn.rn50_recipe_hparams_transition(epoch, kind)
            eta = orc.lr_slow_start(epoch)
            a = orc.alpha_sgd_transition(epoch, kind)
            assert hp.eta == np.float32(eta) and hp.a_sgd == np.float32(a)
            assert hp.a_rms == np.float32(orc.alpha_rmsprop(a, 3e-4, eta))
    ref, hp = rn.rn50_recipe_hparams(7.0), rn.rn50_recipe_hparams_transition(7.0, rn.TRANSITION_ELU)
    assert (ref.eta, ref.a_sgd, ref.a_rms) == (hp.eta, hp.a_sgd, hp.a_rms)
    sudden = rn.rn50_recipe_hparams_transition(9.0, rn.TRANSITION_SUDDEN)
    assert sudden.a_sgd == 0.0 and abs(sudden.eta * sudden.a_rms - 3e-4) < 1e-9       # pure RMSprop before the switch
    assert rn.lib().rn50_recipe_hparams_transition(1.0, 1024, 32, 4, C.byref(hp)) == rn.EINVAL
    assert rn.lib().rn50_recipe_hparams_transition(1.0, 1024, 32, -1, C.byref(hp)) == rn.EINVAL


def test_workspace_sizes_are_consistent():
    for name, c, k, r, stride, pad, h in resnet50.conv_layers():
        d = rn.conv_desc(32, c, h, h, k, r, r, stride, pad)
        for op in (rn.OP_FWD, rn.OP_BWD_DATA, rn.OP_BWD_WEIGHT):
            b = rn.rn50_conv_workspace_bytes(d, op)
            assert 0 <= b < 2 << 30, (name, op, b)
        assert rn.rn50_conv_workspace_bytes(d, rn.OP_BWD_WEIGHT) >= 4 * k * c * r * r
    assert rn.rn50_bn_workspace_bytes(32, 64, 112, 112) > 0
    assert rn.rn50_bn_workspace_bytes(32, 6, 4, 4) == 0
    a32, a64 = rn.rn50_activation_bytes(32), rn.rn50_activation_bytes(64)
    assert 2e9 < a32 < 8e9 and a32 < a64 < 2.1 * a32
    assert rn.rn50_activation_bytes(0) == 0


def test_two_call_data_gradient_argument_errors():
    L = rn.lib()
    d = rn.conv_desc(2, 64, 8, 8, 64, 3, 3, 1, 1)
    assert L.conv2d_filter_flip(C.byref(d), None, 16, None) == rn.EINVAL
    assert L.conv2d_filter_flip(C.byref(d), 16, 16, None) == rn.EINVAL             # in place
    assert L.conv2d_filter_flip(C.byref(d), 16, 36, None) == rn.EINVAL             # misaligned
    assert L.conv2d_bwd_data_flipped(C.byref(d), None, 16, 32, None, 0, None) == rn.EINVAL
    forced = rn.conv_desc(2, 64, 8, 8, 64, 3, 3, 1, 1)
    rn.rn50_set_option("igemm_plan", "64,64,3")                                    # a plan with partial tiles: workspace needed
    try:
        need = rn.rn50_conv_workspace_bytes(forced, rn.OP_BWD_DATA_FLIPPED)
        assert need > 0
        assert L.conv2d_bwd_data_flipped(C.byref(forced), 16, 32, 48, 64, need - 1, None) == rn.EWORKSPACE
    finally:
        rn.rn50_set_option("igemm_plan", None)
    assert L.rn50_filter_flip_all(None, 16, None) == rn.EINVAL


def test_plan_overrides_go_before_the_table():
    """Rows of the "plan_overrides" option replace the plan of exactly the (direction, shape) they name; seen through the workspace
    size, which is the number of partial tiles (implicit GEMM) or of partial filters (filter gradient) of the plan."""
    d = rn.conv_desc(32, 256, 14, 14, 256, 3, 3, 1, 1)       # a tuned shape: 6272 x 256 outputs, reduction 2304
    other = rn.conv_desc(32, 128, 28, 28, 128, 3, 3, 1, 1)
    base = {op: rn.rn50_conv_workspace_bytes(d, op) for op in (rn.OP_FWD, rn.OP_BWD_WEIGHT)}
    base_other = rn.rn50_conv_workspace_bytes(other, rn.OP_FWD)
    # forward as 64x64 tiles cut into 3 pieces: 98 x 4 tiles, all in the split tail (fewer tiles than the chip holds)
    rn.rn50_set_option("plan_overrides", "0,32,256,14,256,3,1,1,64,64,3;2,32,256,14,256,3,1,1,128,128,7;junk")
    assert rn.rn50_conv_workspace_bytes(d, rn.OP_FWD) == 98 * 4 * 3 * 64 * 64 * 4
    assert rn.rn50_conv_workspace_bytes(d, rn.OP_BWD_WEIGHT) == 7 * 256 * 2304 * 4
    assert rn.rn50_conv_workspace_bytes(other, rn.OP_FWD) == base_other
    rn.rn50_set_option("plan_overrides", "0,32,256,14,256,3,1,1,64,64,1")
    assert rn.rn50_conv_workspace_bytes(d, rn.OP_FWD) == 0
    assert rn.rn50_conv_workspace_bytes(d, rn.OP_BWD_WEIGHT) == base[rn.OP_BWD_WEIGHT]
    rn.rn50_set_option("plan_overrides", "0,32,256,14,256,3,1,1,96,64,3")      # not a tile shape: row ignored
    assert rn.rn50_conv_workspace_bytes(d, rn.OP_FWD) == base[rn.OP_FWD]
    rn.rn50_set_option("plan_overrides", None)
    assert rn.rn50_conv_workspace_bytes(d, rn.OP_FWD) == base[rn.OP_FWD]


def test_validation_happens_before_any_gpu_call():
    L = rn.lib()
    hp = rn.opt_hparams(0.1)
    assert L.opt_update(64, 16, 16, 16, None, None, None, C.byref(hp), None) == rn.EINVAL
    assert b"exactly one" in L.rn50_last_error()
    assert L.opt_update(64, 16, 16, 17, 16, None, None, C.byref(hp), None) == rn.EINVAL      # misaligned
    assert L.grad_pack_fp16(8, None, 16, None) == rn.EINVAL
    assert L.grad_pack_fp16(0, None, None, None) == rn.OK                                    # empty input: nothing to do
    d = rn.conv_desc(1, 8, 4, 4, 8, 3, 3, 1, 1, layout=rn.LAYOUT_NCHW)
    assert L.conv2d_fwd(C.byref(d), 16, 16, 16, None, 0, None) == rn.EUNSUPPORTED
    d = rn.conv_desc(1, 8, 4, 4, 8, 3, 3, 0, 1)
    assert L.conv2d_fwd(C.byref(d), 16, 16, 16, None, 0, None) == rn.EINVAL
    d = rn.conv_desc(32, 64, 56, 56, 64, 3, 3, 1, 1)
    assert L.conv2d_bwd_weight(C.byref(d), 16, 16, 16, 16, 16, None) == rn.EWORKSPACE
    assert L.conv2d_fwd(None, 16, 16, 16, None, 0, None) == rn.EINVAL
    assert L.bn_fwd_batchstats(1, 6, 2, 2, rn.LAYOUT_NHWC, 16, 16, 16, 1e-5, None, 0, 16, 16, 16, 16, 1 << 20, None) == rn.EUNSUPPORTED
    assert L.bn_bwd_batchstats(1, 8, 2, 2, rn.LAYOUT_NHWC, 16, 16, None, None, 16, 16, 16, 1, 16, None, 16, 16, 16, 1 << 20, None) == rn.EINVAL
    # the calls whose input is a BN + ReLU applied on the fly, the statistics-only BN and the byte-mask BN
    d = rn.conv_desc(1, 20, 8, 8, 24, 3, 3, 1, 1)
    assert L.conv2d_fwd_bnrelu_input(C.byref(d), 16, 16, 16, 16, 16, 16, 1 << 20, None) == rn.EUNSUPPORTED   # C % 32 != 0
    d = rn.conv_desc(1, 32, 8, 8, 32, 3, 3, 1, 1)
    assert L.conv2d_fwd_bnrelu_input(C.byref(d), 16, None, 16, 16, 16, 16, 1 << 20, None) == rn.EINVAL
    assert L.conv2d_fwd_bnrelu_input(C.byref(d), 16, 16, 20, 16, 16, 16, 1 << 20, None) == rn.EINVAL               # misaligned shift
    assert L.conv2d_bwd_weight_bnrelu_input(C.byref(d), 16, 16, None, 16, 16, 16, 1 << 20, None) == rn.EINVAL
    assert L.conv2d_bwd_weight_bnrelu_input(C.byref(d), 16, 16, 16, 16, 16, 16, 64, None) == rn.EWORKSPACE
    assert L.conv2d_fwd_bnrelu_input(None, 16, 16, 16, 16, 16, 16, 0, None) in (rn.EINVAL, rn.EUNSUPPORTED)
    assert L.maxpool3x3s2_fwd_bnrelu_input(1, 8, 4, 4, 16, None, 16, 16, 16, None) == rn.EINVAL
    assert L.maxpool3x3s2_fwd_bnrelu_input(1, 6, 4, 4, 16, 16, 16, 16, 16, None) == rn.EUNSUPPORTED
    assert L.bn_stats_scale_shift(1, 8, 2, 2, rn.LAYOUT_NHWC, 16, 16, 16, 1e-5, 16, 16, None, 16, 16, 1 << 20, None) == rn.EINVAL
    assert L.bn_stats_scale_shift(1, 8, 2, 2, rn.LAYOUT_NHWC, 16, 16, 16, 1e-5, 16, 16, 16, 16, 16, 16, None) == rn.EWORKSPACE
    assert L.bn_fwd_batchstats_mask(1, 8, 2, 2, rn.LAYOUT_NHWC, 16, 16, 16, 1e-5, None, 16, None, 16, 16, 16, 1 << 20, None) == rn.EINVAL
    assert L.bn_bwd_batchstats_mask(1, 8, 2, 2, rn.LAYOUT_NHWC, 16, 16, None, None, 16, 16, 16, 16, None, 16, 16, 16, 1 << 20, None) == rn.EINVAL
    assert L.softmax_ce(2000, 10, 16, 16, 16, 16, None) == rn.EUNSUPPORTED
    assert L.fc_fwd(2, 6, 3, 16, 16, 16, 16, None) == rn.EUNSUPPORTED
    h = C.c_void_p()
    assert L.rn50_create(C.byref(h), 32, 7, 0, 256, 1 << 40) == rn.EINVAL                      # unknown variant
    assert L.rn50_activation_bytes(32, 7) == 0
    assert L.rn50_activation_bytes(32, rn.VARIANT_V15) > L.rn50_activation_bytes(32, rn.VARIANT_V1) > 0
    assert L.rn50_create(C.byref(h), 32, 0, 9, 256, 1 << 40) == rn.EINVAL                      # unknown operand dtype
    assert L.rn50_create(C.byref(h), 32, 0, 0, 256, 1024) == rn.EWORKSPACE
    assert L.rn50_create(C.byref(h), 32, 0, 0, 100, 1 << 40) == rn.EINVAL                      # misaligned arena
    assert L.rn50_param_table(999, None, None, None, None, None) == rn.EINVAL
    # the measurement probes check their arguments the same way
    assert L.rn50_probe_mfma(7, 1, 1, 16, None, None, None) == rn.EINVAL                      # unknown dtype
    assert L.rn50_probe_mfma(rn.DTYPE_F32, 0, 1, 16, None, None, None) == rn.EINVAL
    assert L.rn50_probe_mfma(rn.DTYPE_F32, 1, 9, 16, None, None, None) == rn.EINVAL
    assert L.rn50_probe_mfma(rn.DTYPE_F32, 1, 1, None, None, None, None) == rn.EINVAL
    assert L.rn50_probe_mfma(rn.DTYPE_F32, 1, 1, 16, 20, None, None) == rn.EINVAL             # misaligned tick buffer
    assert L.rn50_probe_copy(6, 16, 32, None) == rn.EINVAL                                    # not a multiple of 4
    assert L.rn50_probe_copy(8, None, 32, None) == rn.EINVAL
    assert L.rn50_probe_empty(0, 1, None, None) == rn.EINVAL
    assert L.rn50_probe_empty(1, 0, None, None) == rn.EINVAL


def test_recipe_hparams_follow_the_paper_schedules():
    """Appendix A.1 / A.2 scalars of one iteration, against the oracle's schedule functions and the printed constants."""
    from oracle import ops as orc
    for epoch in (0.0, 3.3, 5.0, 9.99, 10.0, 11.25, 12.5, 20.0, 39.99, 40.0, 69.0, 70.0, 84.9, 85.0, 89.9):
        hp = rn.rn50_recipe_hparams(epoch)
        eta = orc.lr_slow_start(epoch)
        a = orc.alpha_sgd(epoch)
        assert hp.eta == np.float32(eta)
        assert hp.a_sgd == np.float32(a)
        assert hp.a_rms == np.float32(orc.alpha_rmsprop(a, 3e-4, eta))
        assert (hp.mu1, hp.mu2, hp.eps, hp.wd, hp.g_scale) == (np.float32(0.9), np.float32(0.99), np.float32(1e-8), np.float32(1e-4), 1.0 / 1024)
    hp = rn.rn50_recipe_hparams(0.0)
    assert abs(hp.eta - 6.4) < 1e-6 and abs(hp.a_sgd - 0.5 * math.exp(-4)) < 1e-9     # Appendix A.2: 6.4 until epoch 40
    assert abs(hp.eta * hp.a_rms - (1 - hp.a_sgd) * 3e-4) < 1e-9                        # eta * alpha_RMSprop = (1 - alpha_SGD) * eta_RMSprop
    one = rn.rn50_recipe_hparams(0.0, 1, 32)
    assert abs(one.eta - 0.5 * 0.0125) < 1e-9 and one.g_scale == 1.0
    L = rn.lib()
    assert L.rn50_recipe_hparams(-1.0, 1024, 32, C.byref(hp)) == rn.EINVAL
    assert L.rn50_recipe_hparams(1.0, 0, 32, C.byref(hp)) == rn.EINVAL
    assert L.rn50_recipe_hparams(1.0, 1024, 32, None) == rn.EINVAL


def test_options_are_a_snapshot_replaced_as_a_whole():
    """rn50_set_option: unknown names and malformed plans are rejected and leave the snapshot as it was; NULL restores the
    default; the plan a call uses is the one in force when it starts (seen through the workspace size)."""
    L = rn.lib()
    d = rn.conv_desc(2, 64, 8, 8, 64, 3, 3, 1, 1)
    base = rn.rn50_conv_workspace_bytes(d, rn.OP_BWD_WEIGHT)
    assert L.rn50_set_option(None, b"1") == rn.EINVAL
    assert L.rn50_set_option(b"no_such_switch", b"1") == rn.EINVAL
    assert b"no_such_switch" in L.rn50_last_error()
    assert L.rn50_set_option(b"wgrad_plan", b"96,64,2") == rn.EINVAL          # 96 is not a tile edge
    assert rn.rn50_conv_workspace_bytes(d, rn.OP_BWD_WEIGHT) == base
    rn.rn50_set_option("wgrad_plan", "64,64,1")                               # one range: one partial of the 64 x 576 gradient
    assert rn.rn50_conv_workspace_bytes(d, rn.OP_BWD_WEIGHT) == 64 * 64 * 9 * 4 != base
    rn.rn50_set_option("wgrad_plan", "")
    assert rn.rn50_conv_workspace_bytes(d, rn.OP_BWD_WEIGHT) == base
    for name in ("side_stream", "fuse_bn", "relu_mask", "no_tuned", "no_stem_kernel"):
        rn.rn50_set_option(name, "1")
        rn.rn50_set_option(name, None)
    tuned = rn.conv_desc(32, 256, 14, 14, 256, 3, 3, 1, 1)
    with_table = rn.rn50_conv_workspace_bytes(tuned, rn.OP_BWD_WEIGHT)
    rn.rn50_set_option("no_tuned", "1")
    try:
        assert rn.rn50_conv_workspace_bytes(tuned, rn.OP_BWD_WEIGHT) > 0      # cost model in force; any positive size
    finally:
        rn.rn50_set_option("no_tuned", None)
    assert rn.rn50_conv_workspace_bytes(tuned, rn.OP_BWD_WEIGHT) == with_table


def test_conv_fwd_bnstats_argument_errors():
    L = rn.lib()
    d0 = rn.conv_desc(32, 256, 14, 14, 256, 3, 3, 1, 1)
    assert rn.rn50_conv_plan(d0, rn.OP_FWD_BNSTATS) == rn.rn50_conv_plan(d0, rn.OP_FWD)
    d = rn.conv_desc(2, 64, 8, 8, 64, 3, 3, 1, 1)
    need = rn.rn50_conv_workspace_bytes(d, rn.OP_FWD_BNSTATS)
    assert need >= rn.rn50_conv_workspace_bytes(d, rn.OP_FWD) + 2 * 2 * 64 * 4
    a = [16] * 4
    assert L.conv2d_fwd_bnstats(C.byref(d), 16, None, None, 16, 16, 16, 16, 2e-5, *a, 256, need - 1, None) == rn.EWORKSPACE
    assert L.conv2d_fwd_bnstats(C.byref(d), 16, 16, None, 16, 16, 16, 16, 2e-5, *a, 256, need, None) == rn.EINVAL   # scale without shift
    assert L.conv2d_fwd_bnstats(C.byref(d), 16, None, None, 16, 16, None, 16, 2e-5, *a, 256, need, None) == rn.EINVAL
    assert L.conv2d_fwd_bnstats(C.byref(d), 16, None, None, 16, 16, 16, 16, -1.0, *a, 256, need, None) == rn.EINVAL
    assert L.conv2d_fwd_bnstats(C.byref(d), None, None, None, 16, 16, 16, 16, 2e-5, *a, 256, need, None) == rn.EINVAL
    d2 = rn.conv_desc(2, 64, 8, 8, 30, 3, 3, 1, 1)
    assert L.conv2d_fwd_bnstats(C.byref(d2), 16, None, None, 16, 16, 16, 16, 2e-5, *a, 256, 1 << 30, None) == rn.EUNSUPPORTED
    d3 = rn.conv_desc(2, 20, 8, 8, 64, 3, 3, 1, 1)
    assert L.conv2d_fwd_bnstats(C.byref(d3), 16, 16, 16, 16, 16, 16, 16, 2e-5, *a, 256, 1 << 30, None) == rn.EUNSUPPORTED
    assert L.bn_fwd_apply(1, 8, 2, 2, rn.LAYOUT_NHWC, 16, 16, None, None, 0, 16, None, None) == rn.EINVAL
    assert L.bn_fwd_apply(1, 8, 2, 2, rn.LAYOUT_NHWC, 16, 16, 16, None, 0, 16, 16, None) == rn.EINVAL             # mask without ReLU
    assert L.bn_fwd_apply(1, 6, 2, 2, rn.LAYOUT_NHWC, 16, 16, 16, None, 0, 16, None, None) == rn.EUNSUPPORTED


def test_wgrad_group_plan_on_the_host():
    """rn50_wgrad_group_plan writes its plan into host memory and touches no device: sizes, error paths and the effect of the
    work-item length on the workspace can be checked without a GPU (device pointers are stand-ins that are never followed)."""
    d1 = rn.conv_desc(32, 64, 56, 56, 256, 1, 1, 1, 0)     # 100352 pixels = 3136 stages
    d2 = rn.conv_desc(32, 512, 7, 7, 512, 3, 3, 1, 1)      # 1568 pixels = 49 stages
    fake = 4096

    def items(descs, off_step=1 << 24):
        arr = (rn.WgradGroupItem * len(descs))()
        for i, (it, d) in enumerate(zip(arr, descs)):
            it.desc, it.x, it.in_scale, it.in_shift, it.dy, it.dw_offset = d, fake, None, None, fake, i * off_step
        return arr

    L = rn.lib()
    assert rn.rn50_wgrad_group_table_bytes(0) == 0 and rn.rn50_wgrad_group_table_bytes(2) > rn.rn50_wgrad_group_table_bytes(1) > 0
    rn.rn50_set_option("wgrad_group_stages", "32")
    try:
        it = items([d1, d2])
        need = rn.rn50_wgrad_group_workspace_bytes(it)
        # 3136 stages in 98 ranges of 32; 49 stages in 2 ranges (26 + 23: ranges take an even number of stages)
        assert need == 4 * (98 * 256 * 64 + 2 * 512 * 9 * 512)
        table = C.create_string_buffer(rn.rn50_wgrad_group_table_bytes(2))
        assert L.rn50_wgrad_group_plan(2, it, fake, need, table, len(table)) == rn.OK
        assert L.rn50_wgrad_group_plan(2, it, fake, need - 4, table, len(table)) == rn.EWORKSPACE
        assert L.rn50_wgrad_group_plan(2, it, fake, need, table, len(table) - 1) == rn.EINVAL
        assert L.rn50_wgrad_group_plan(2, it, None, need, table, len(table)) == rn.EINVAL
        assert L.rn50_wgrad_group_plan(0, it, fake, need, table, len(table)) == rn.EINVAL
        rn.rn50_set_option("wgrad_group_stages", "64")
        assert rn.rn50_wgrad_group_workspace_bytes(it) == 4 * (49 * 256 * 64 + 1 * 512 * 9 * 512)
    finally:
        rn.rn50_set_option("wgrad_group_stages", None)
    bad = items([rn.conv_desc(32, 3, 224, 224, 64, 7, 7, 2, 3)])       # C % 4 != 0: the first layer is not for this call
    assert rn.rn50_wgrad_group_workspace_bytes(bad) == 0
    assert L.rn50_wgrad_group_plan(1, bad, fake, 1 << 30, table, len(table)) == rn.EUNSUPPORTED
    bf = items([rn.conv_desc(32, 64, 56, 56, 64, 1, 1, 1, 0, in_dtype=rn.DTYPE_BF16)])
    assert L.rn50_wgrad_group_plan(1, bf, fake, 1 << 30, table, len(table)) == rn.EUNSUPPORTED
    assert L.conv2d_bwd_weight_group(None, fake, fake, None) == rn.EINVAL
    junk = C.create_string_buffer(len(table))
    assert L.conv2d_bwd_weight_group(junk, fake, fake, None) == rn.EINVAL    # not a plan: nothing is launched
    assert L.rn50_wgrad_groups_run(None, fake, None) == rn.EINVAL
