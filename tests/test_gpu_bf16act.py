"""GPU parity of the variant that keeps activations as bfloat16 in memory (RN50_DTYPE_BF16_ACT).

Every tensor a call reads holds bf16-representable values (the test rounds its seeded inputs with a frexp / rint routine
that shares nothing with the kernels' integer bit arithmetic), so the oracle sees exactly the operands the kernel sees;
the oracle computes in fp64 and the device result, which is the fp32 result rounded to bf16 at the store, is held to
  - the variant's stated tolerance against the oracle's unrounded result (rel-L2 <= 1e-2; bf16 rounding alone is ~1.5e-3),
  - and, much tighter, against the oracle's result rounded to bf16: at most one bf16 step apart anywhere, and different at
    all only where the fp32 and fp64 sums fall on two sides of a rounding boundary (a small fraction of the elements).
Filter gradients, BN statistics and parameter gradients stay fp32 and meet the fp32 bar of 1e-4.
"""
import math

import numpy as np
import pytest
import torch

from oracle import ops as orc
from oracle import resnet50
from paper_1711_04325_amd import binding as rn
from paper_1711_04325_amd import synth
from tests.gpu_util import DEV, TOL, assert_close, bf16_round, empty, nchw, nhwc, rel_l2, to_dev, ws_bytes
from tests.step_util import dict_from_flat, flat_from_dict, gpu_forward_backward, problem

pytestmark = pytest.mark.gpu
BN_EPS = 2e-5
ACT, F32IN = rn.DTYPE_BF16_ACT, rn.DTYPE_BF16_ACT_F32IN


def r16(a):
    """Seeded values rounded to bf16 (float32 array)."""
    return bf16_round(a).astype(np.float32)


def h_nhwc(a):
    """logical NCHW array of bf16-representable values -> device NHWC bfloat16 tensor (exact)."""
    return nhwc(a).to(torch.bfloat16).contiguous()


def h_empty(*shape):
    return torch.empty(shape, dtype=torch.bfloat16, device=DEV)


def h_nchw(t):
    return np.transpose(t.float().cpu().numpy().astype(np.float64), (0, 3, 1, 2))


def assert_bf16(got, ref, what, frac=5e-3):
    """got: device values (bf16-representable, float64 array); ref: the oracle's fp64 result."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert np.all(np.isfinite(got)), what
    e_raw = rel_l2(got, ref)
    assert e_raw <= 1e-2, "%s: rel-L2 %.2e against the unrounded oracle" % (what, e_raw)
    r = bf16_round(ref)
    diff = np.abs(got - r)
    # one bf16 step is at most 2^-7 of the magnitude; an element that cancelled to nearly nothing carries the fp32 summation
    # error of its terms, which can exceed its own tiny step: allow 1e-5 of the tensor's r.m.s. on top
    step = np.maximum(np.abs(r), np.abs(got)) * 2.0 ** -7 + 1e-5 * np.sqrt(np.mean(ref * ref)) + 1e-30
    assert np.all(diff <= step), "%s: %d elements more than one bf16 step from the rounded oracle" % (what, int(np.sum(diff > step)))
    f = float(np.mean(diff > 0))
    assert f <= frac, "%s: %.2e of the elements differ from the rounded oracle" % (what, f)
    e = rel_l2(got, r)
    assert e <= 1e-3, "%s: rel-L2 %.2e against the rounded oracle" % (what, e)
    return e_raw, f


# ------------------------------------------------------------------------------------------------------------------
# convolutions
# ------------------------------------------------------------------------------------------------------------------
CONV_CASES = [
    (2, 64, 56, 56, 64, 1, 1, 0),
    (2, 64, 28, 28, 64, 3, 1, 1),
    (2, 64, 56, 56, 256, 1, 1, 0),
    (3, 256, 14, 14, 64, 1, 1, 0),    # ragged row tiles
    (2, 128, 28, 28, 96, 1, 2, 0),    # 1x1 stride 2: scatter epilogue in the data gradient; K = 96
    (1, 32, 9, 11, 40, 3, 1, 1),      # odd sizes
    (2, 512, 7, 7, 512, 3, 1, 1),     # long reduction: split tails
    (2, 64, 16, 16, 64, 3, 2, 1),     # 3x3 stride 2, even input: parity-class row order in the data gradient
    (2, 64, 15, 15, 64, 3, 2, 1),     # 3x3 stride 2, odd input
    (2, 1024, 7, 7, 2048, 1, 1, 0),
    (1, 24, 8, 8, 24, 3, 1, 1),       # channel count that is not a multiple of 32: scalar gather of bf16
]


def _conv_all(case, seed, dtype=ACT):
    n, c, h, w, k, r, stride, pad = case
    g = synth.rng(seed)
    x = synth.normal(g, (n, c, h, w))
    x = x if dtype == F32IN else r16(x)
    wt = synth.he_normal(g, (k, c, r, r))
    p, q = orc.out_size(h, r, stride, pad), orc.out_size(w, r, stride, pad)
    dy = r16(synth.normal(g, (n, k, p, q)))
    d = rn.conv_desc(n, c, h, w, k, r, r, stride, pad, in_dtype=dtype)
    dx_ = nhwc(x) if dtype == F32IN else h_nhwc(x)
    dw_, ddy_ = nhwc(wt), h_nhwc(dy)
    y = h_empty(n, p, q, k)
    rn.conv2d_fwd(d, dx_, dw_, y, ws_bytes(rn.rn50_conv_workspace_bytes(d, rn.OP_FWD)))
    gdw = empty(k, r, r, c)
    rn.conv2d_bwd_weight(d, dx_, ddy_, gdw, ws_bytes(rn.rn50_conv_workspace_bytes(d, rn.OP_BWD_WEIGHT)))
    gdx = None
    if dtype == ACT:
        gdx = torch.full((n, h, w, c), float("nan"), dtype=torch.bfloat16, device=DEV)
        rn.conv2d_bwd_data(d, ddy_, dw_, gdx, ws_bytes(rn.rn50_conv_workspace_bytes(d, rn.OP_BWD_DATA)))
    torch.cuda.synchronize()
    xo, wo = bf16_round(x), bf16_round(wt)         # the operands the MFMAs see
    assert_bf16(h_nchw(y), orc.conv2d_fwd(xo, wo, stride, pad), "fwd %s" % (case,))
    assert_close(nchw(gdw), orc.conv2d_bwd_weight(xo, dy, r, r, stride, pad), TOL, "bwd_weight %s" % (case,))
    if gdx is not None:
        assert_bf16(h_nchw(gdx), orc.conv2d_bwd_data(dy, wo, stride, pad, h, w), "bwd_data %s" % (case,))
    return y, gdw, gdx


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_bf16_activations(case):
    rn.rn50_set_option("igemm_plan", None)
    rn.rn50_set_option("wgrad_plan", None)
    _conv_all(case, 600 + CONV_CASES.index(case))


@pytest.mark.parametrize("plan", ["128,128,1", "128,64,1", "64,128,1", "64,64,1", "128,128,3", "64,64,4", "64,128,2"])
@pytest.mark.parametrize("case", [CONV_CASES[1], CONV_CASES[3], CONV_CASES[6], CONV_CASES[7], CONV_CASES[10]])
def test_conv_bf16_activations_every_tile_shape_and_split(case, plan):
    rn.rn50_set_option("igemm_plan", plan)
    rn.rn50_set_option("wgrad_plan", plan.rsplit(",", 1)[0] + "," + str(int(plan.rsplit(",", 1)[1]) * 5))   # tile is 64x64 whatever is asked
    try:
        _conv_all(case, 7)
    finally:
        rn.rn50_set_option("igemm_plan", None)
        rn.rn50_set_option("wgrad_plan", None)


def act_plan_shapes():
    """Unique (n, c, h, w, k, r, stride, pad) of the plan table measured for this storage, with the directions that have a row."""
    import os
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    txt = open(os.path.join(root, "paper_1711_04325_amd", "csrc", "conv_plans_bf16act.inc")).read()
    seen = {}
    for m in re.finditer(r"^\s*\{([-0-9, ]+)\},", txt, flags=re.M):
        op, n, c, h, k, r, stride, pad, bm, bn, split = (int(v) for v in m.group(1).split(","))
        seen.setdefault((n, c, h, h, k, r, stride, pad), set()).add(op)
    return sorted(seen.items())


ACT_SWEEP = act_plan_shapes()


@pytest.mark.parametrize("case,ops", ACT_SWEEP, ids=["n%d_c%d_h%d_k%d_r%d_s%d" % (c[0], c[1], c[2], c[4], c[5], c[6]) for c, _ in ACT_SWEEP])
def test_bf16_activation_plan_rows_on_sampled_outputs(case, ops):
    """Every row of the plan table of this storage, launched with the shape it was measured for and graded on outputs the oracle
    computes one by one: three whole images of the convolution and of its data gradient (bf16 tensors: one-bf16-step bar), two
    whole output channels of the filter gradient over every image and pixel (fp32: 1e-4)."""
    rn.rn50_set_option("igemm_plan", None)
    rn.rn50_set_option("wgrad_plan", None)
    n, c, h, w, k, r, stride, pad = case
    first = c == 3
    g = synth.rng(2000 + sum(case))
    x = synth.normal(g, (n, c, h, w))
    if not first:
        x = r16(x)
    wt = synth.he_normal(g, (k, c, r, r))
    p, q = orc.out_size(h, r, stride, pad), orc.out_size(w, r, stride, pad)
    dy = r16(synth.normal(g, (n, k, p, q)))
    d = rn.conv_desc(n, c, h, w, k, r, r, stride, pad, in_dtype=F32IN if first else ACT)
    dx_ = nhwc(x) if first else h_nhwc(x)
    dw_, ddy_ = nhwc(wt), h_nhwc(dy)
    imgs, chans = [0, n // 2, n - 1], [0, k - 1]
    xo, wo = bf16_round(x), bf16_round(wt)
    y = h_empty(n, p, q, k)
    rn.conv2d_fwd(d, dx_, dw_, y, ws_bytes(rn.rn50_conv_workspace_bytes(d, rn.OP_FWD)))
    gdw = empty(k, r, r, c)
    rn.conv2d_bwd_weight(d, dx_, ddy_, gdw, ws_bytes(rn.rn50_conv_workspace_bytes(d, rn.OP_BWD_WEIGHT)))
    torch.cuda.synchronize()
    what = str(case)
    got_y = np.transpose(y[imgs].float().cpu().numpy().astype(np.float64), (0, 3, 1, 2))
    assert_bf16(got_y, orc.conv2d_fwd(xo[imgs], wo, stride, pad), "fwd " + what)
    assert bool(torch.isfinite(y.float()).all()), "fwd " + what
    del y
    got_dw = np.transpose(gdw[chans].cpu().numpy().astype(np.float64), (0, 3, 1, 2))
    assert_close(got_dw, orc.conv2d_bwd_weight(xo, np.ascontiguousarray(dy[:, chans]), r, r, stride, pad), TOL, "bwd_weight " + what)
    assert bool(torch.isfinite(gdw).all()), "bwd_weight " + what
    if 1 in ops:
        gdx = torch.full((n, h, w, c), float("nan"), dtype=torch.bfloat16, device=DEV)
        rn.conv2d_bwd_data(d, ddy_, dw_, gdx, ws_bytes(rn.rn50_conv_workspace_bytes(d, rn.OP_BWD_DATA)))
        torch.cuda.synchronize()
        got_dx = np.transpose(gdx[imgs].float().cpu().numpy().astype(np.float64), (0, 3, 1, 2))
        assert_bf16(got_dx, orc.conv2d_bwd_data(dy[imgs], wo, stride, pad, h, w), "bwd_data " + what)
        assert bool(torch.isfinite(gdx.float()).all()), "bwd_data " + what


@pytest.mark.parametrize("case", [(2, 3, 64, 64, 64, 7, 2, 3), (1, 3, 50, 38, 64, 7, 2, 3), (2, 32, 12, 12, 64, 3, 1, 1)])
def test_conv_bf16_activations_with_an_fp32_input(case):
    """The network's first layer: the image is fp32 (rounded on the way into LDS), output and incoming gradient are bf16."""
    _conv_all(case, 650 + sum(case), dtype=F32IN)
    d = rn.conv_desc(*case[:5], case[5], case[5], case[6], case[7], in_dtype=F32IN)
    t = empty(64)
    with pytest.raises(rn.Rn50Error) as e:
        rn.conv2d_bwd_data(d, t, t, t, ws_bytes(1 << 22))
    assert e.value.code == rn.EUNSUPPORTED


def test_conv_bf16_activations_is_deterministic_and_checks_arguments():
    a = _conv_all(CONV_CASES[6], 3)
    b = _conv_all(CONV_CASES[6], 3)
    for u, v in zip(a, b):
        assert torch.equal(u.float(), v.float())
    t = empty(4096)
    d = rn.conv_desc(1, 20, 8, 8, 24, 3, 3, 1, 1, in_dtype=ACT)     # 20 channels: the filter gradient needs C % 8 == 0
    with pytest.raises(rn.Rn50Error) as e:
        rn.conv2d_bwd_weight(d, t, t, t, ws_bytes(1 << 20))
    assert e.value.code == rn.EUNSUPPORTED
    d = rn.conv_desc(1, 24, 8, 8, 20, 3, 3, 1, 1, in_dtype=ACT)     # K % 8 != 0
    with pytest.raises(rn.Rn50Error) as e:
        rn.conv2d_bwd_weight(d, t, t, t, ws_bytes(1 << 20))
    assert e.value.code == rn.EUNSUPPORTED


@pytest.mark.parametrize("plan", [None, "128,128,1", "64,128,2", "64,64,3"])
@pytest.mark.parametrize("case", [CONV_CASES[1], CONV_CASES[3], CONV_CASES[6], CONV_CASES[9], (2, 128, 28, 28, 128, 3, 2, 1)])
def test_conv_bf16_activations_with_bn_relu_applied_to_the_input(case, plan):
    """conv2d_fwd_bnrelu_input / conv2d_bwd_weight_bnrelu_input on a bf16 input: max(0, x*scale + shift) formed in fp32 and rounded
    once, i.e. the tensor a normalising kernel would have stored; the unfused calls on that tensor give the same bits."""
    n, c, h, w, k, r, stride, pad = case
    g = synth.rng(41 + sum(case))
    x = r16(synth.normal(g, (n, c, h, w)))
    scale = g.uniform(0.5, 1.5, c).astype(np.float32) * np.where(g.uniform(size=c) < 0.2, -1, 1).astype(np.float32)
    shift = synth.normal(g, c, 0.5) + np.float32(0.3)
    wt = synth.he_normal(g, (k, c, r, r))
    p, q = orc.out_size(h, r, stride, pad), orc.out_size(w, r, stride, pad)
    dy = r16(synth.normal(g, (n, k, p, q)))
    # one fused multiply-add in fp32 (exact product and sum rounded once), ReLU, then the bf16 store
    act = r16(np.maximum(np.float32(0), (x.astype(np.float64) * scale[None, :, None, None] + shift[None, :, None, None]).astype(np.float32)))
    d = rn.conv_desc(n, c, h, w, k, r, r, stride, pad, in_dtype=ACT)
    rn.rn50_set_option("igemm_plan", plan)
    rn.rn50_set_option("wgrad_plan", None if plan is None else "64,64," + str(int(plan.rsplit(",", 1)[1]) * 3))
    try:
        y, gdw = h_empty(n, p, q, k), empty(k, r, r, c)
        dsc, dsh = to_dev(scale), to_dev(shift)
        rn.conv2d_fwd_bnrelu_input(d, h_nhwc(x), dsc, dsh, nhwc(wt), y, ws_bytes(rn.rn50_conv_workspace_bytes(d, rn.OP_FWD)))
        rn.conv2d_bwd_weight_bnrelu_input(d, h_nhwc(x), dsc, dsh, h_nhwc(dy), gdw, ws_bytes(rn.rn50_conv_workspace_bytes(d, rn.OP_BWD_WEIGHT)))
        y2, gdw2 = h_empty(n, p, q, k), empty(k, r, r, c)
        rn.conv2d_fwd(d, h_nhwc(act), nhwc(wt), y2, ws_bytes(rn.rn50_conv_workspace_bytes(d, rn.OP_FWD)))
        rn.conv2d_bwd_weight(d, h_nhwc(act), h_nhwc(dy), gdw2, ws_bytes(rn.rn50_conv_workspace_bytes(d, rn.OP_BWD_WEIGHT)))
        torch.cuda.synchronize()
    finally:
        rn.rn50_set_option("igemm_plan", None)
        rn.rn50_set_option("wgrad_plan", None)
    assert_bf16(h_nchw(y), orc.conv2d_fwd(act, bf16_round(wt), stride, pad), "fused fwd %s" % (case,))
    assert_close(nchw(gdw), orc.conv2d_bwd_weight(act, dy, r, r, stride, pad), TOL, "fused bwd_weight %s" % (case,))
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))
    assert torch.equal(gdw, gdw2)


# ------------------------------------------------------------------------------------------------------------------
# batch normalization and pooling
# ------------------------------------------------------------------------------------------------------------------
BN_SHAPES = [(2, 64, 56, 56), (4, 256, 14, 14), (3, 2048, 7, 7), (2, 24, 5, 7), (8, 128, 28, 28)]


@pytest.mark.parametrize("relu,res", [(0, 0), (1, 0), (1, 1), (0, 1)])
@pytest.mark.parametrize("shape", BN_SHAPES)
def test_bn_fwd_bf16(shape, relu, res):
    n, c, h, w = shape
    g = synth.rng(700 + sum(shape) + 2 * relu + res)
    x = r16(synth.normal(g, shape, 1.5, 0.7))
    residual = r16(synth.normal(g, shape)) if res else None
    gamma, beta = synth.normal(g, c, 0.1, 1.0), synth.normal(g, c, 0.1)
    y, mean, inv = h_empty(n, h, w, c), empty(c), empty(c)
    mask = torch.zeros(n * h * w * c // 4, dtype=torch.uint8, device=DEV) if relu else None
    wsb = ws_bytes(rn.rn50_bn_workspace_bytes(n, c, h, w))
    rn.bn_fwd_batchstats_bf16(n, c, h, w, h_nhwc(x), to_dev(gamma), to_dev(beta), BN_EPS, h_nhwc(residual) if res else None, relu, y,
                              mask, mean, inv, wsb)
    sc, sh, mean2, inv2 = empty(c), empty(c), empty(c), empty(c)
    rn.bn_stats_scale_shift_bf16(n, c, h, w, h_nhwc(x), to_dev(gamma), to_dev(beta), BN_EPS, mean2, inv2, sc, sh, wsb)
    torch.cuda.synchronize()
    ry, rmean, rinv = orc.bn_fwd(x, gamma, beta, BN_EPS, residual=residual, relu=bool(relu))
    assert_bf16(h_nchw(y), ry, "bn fwd %s" % (shape,))
    assert_close(mean.cpu().numpy(), rmean, TOL, "mean")
    assert_close(inv.cpu().numpy(), rinv, TOL, "invstd")
    assert torch.equal(mean, mean2) and torch.equal(inv, inv2)
    assert_close(sc.cpu().numpy(), gamma * rinv, TOL, "scale")
    assert_close(sh.cpu().numpy(), beta - rmean * gamma * rinv, 1e-4 + 1e-6, "shift")
    if relu:   # byte mask = sign of the STORED output
        bits = mask.cpu().numpy().reshape(n, h, w, c // 4)
        yy = y.float().cpu().numpy().reshape(n, h, w, c // 4, 4)
        for e in range(4):
            np.testing.assert_array_equal((bits >> e) & 1, (yy[..., e] > 0).astype(np.uint8))


@pytest.mark.parametrize("mode", ["y", "mask", "xmask", "norelu", "two", "two_mask_dres"])
@pytest.mark.parametrize("shape", BN_SHAPES)
def test_bn_bwd_bf16(shape, mode):
    """Saved forward tensors come from the oracle (rounded to bf16 as the forward would store them), so the masks are functions of
    the inputs.  Where the residual gradient is requested, dz is rounded before it is used: the oracle gets the rounded sum."""
    n, c, h, w = shape
    g = synth.rng(800 + sum(shape))
    x = r16(synth.normal(g, shape, 1.5, 0.3))
    gamma, beta = synth.normal(g, c, 0.1, 1.0), synth.normal(g, c, 0.1)
    relu = mode != "norelu"
    ry, rmean, rinv = orc.bn_fwd(x, gamma, beta, BN_EPS, relu=relu)
    # the forward's own arithmetic for the stored output: fp32 scale and shift, one fused multiply-add, ReLU, bf16 store
    m32, i32 = rmean.astype(np.float32), rinv.astype(np.float32)
    sc32 = (gamma * i32).astype(np.float32)
    sh32 = (beta.astype(np.float64) - m32.astype(np.float64) * sc32.astype(np.float64)).astype(np.float32)
    pre = (x.astype(np.float64) * sc32[None, :, None, None] + sh32[None, :, None, None]).astype(np.float32)
    y16 = r16(np.maximum(pre, 0) if relu else pre)
    dy = r16(synth.normal(g, shape))
    dy2 = r16(synth.normal(g, shape)) if mode.startswith("two") else None
    want_res = mode == "two_mask_dres"
    dx, dres = h_empty(n, h, w, c), (h_empty(n, h, w, c) if want_res else None)
    dg, db = empty(c), empty(c)
    wsb = ws_bytes(rn.rn50_bn_workspace_bytes(n, c, h, w))
    yd = h_nhwc(y16)
    mask = None
    if mode in ("mask", "two_mask_dres"):
        bits = (np.transpose(y16, (0, 2, 3, 1)).reshape(n, h, w, c // 4, 4) > 0).astype(np.uint8)
        mask = torch.from_numpy(np.ascontiguousarray(bits[..., 0] | (bits[..., 1] << 1) | (bits[..., 2] << 2) | (bits[..., 3] << 3))).to(DEV)
    rn.bn_bwd_batchstats_bf16(n, c, h, w, h_nhwc(x), h_nhwc(dy), h_nhwc(dy2) if dy2 is not None else None,
                              yd if (relu and mode in ("y", "two")) else None, mask, to_dev(gamma), to_dev(beta) if mode == "xmask" else None,
                              to_dev(m32), to_dev(i32), int(relu), dx, dres, dg, db, wsb)
    torch.cuda.synchronize()
    dsum = dy.astype(np.float64) + (dy2 if dy2 is not None else 0.0)
    if want_res:
        dsum = bf16_round(dsum.astype(np.float32))       # the device adds in fp32, then rounds dz to bf16
    rdx, rdres, rdg, rdb = orc.bn_bwd(x, dsum, y16 if relu else None, gamma, m32, i32, relu=relu, want_dresidual=want_res)
    assert_bf16(h_nchw(dx), rdx, "bn bwd dx %s %s" % (shape, mode))
    assert_close(dg.cpu().numpy(), rdg, TOL, "dgamma")
    assert_close(db.cpu().numpy(), rdb, TOL, "dbeta")
    if want_res:
        np.testing.assert_array_equal(h_nchw(dres), rdres)      # dz is bf16-exact on both sides


def test_bn_bf16_argument_errors():
    t = empty(4096)
    L = rn.lib()
    p = t.data_ptr()
    assert L.bn_fwd_batchstats_bf16(1, 8, 2, 2, rn.LAYOUT_NHWC, p, p, p, 1e-5, None, 0, p, p, p, p, p, 1 << 20, None) == rn.EINVAL   # mask without ReLU
    assert L.bn_fwd_batchstats_bf16(1, 6, 2, 2, rn.LAYOUT_NHWC, p, p, p, 1e-5, None, 0, p, None, p, p, p, 1 << 20, None) == rn.EUNSUPPORTED
    # ReLU mask with nothing to take it from; rebuilt from x but a second gradient given
    assert L.bn_bwd_batchstats_bf16(1, 8, 2, 2, rn.LAYOUT_NHWC, p, p, None, None, None, p, None, p, p, 1, p, None, p, p, p, 1 << 20, None) == rn.EINVAL
    assert L.bn_bwd_batchstats_bf16(1, 8, 2, 2, rn.LAYOUT_NHWC, p, p, p, None, None, p, p, p, p, 1, p, None, p, p, p, 1 << 20, None) == rn.EINVAL
    assert L.maxpool3x3s2_fwd_bf16(1, 8, 4, 4, p, p, None, p, p, None) == rn.EINVAL          # scale without shift
    assert L.avgpool_fwd_bf16(1, 6, 4, 4, p, p, None) == rn.EUNSUPPORTED


@pytest.mark.parametrize("shape", [(2, 64, 12, 12), (1, 8, 7, 9), (3, 32, 16, 10)])
def test_pooling_bf16(shape):
    n, c, h, w = shape
    g = synth.rng(900 + sum(shape))
    x = r16(np.maximum(synth.normal(g, shape), 0))           # post-ReLU values: ties at zero
    p, q = (h - 1) // 2 + 1, (w - 1) // 2 + 1
    y, arg = h_empty(n, p, q, c), torch.empty((n, p, q, c), dtype=torch.uint8, device=DEV)
    rn.maxpool3x3s2_fwd_bf16(n, c, h, w, h_nhwc(x), None, None, y, arg)
    ry, rarg = orc.maxpool_fwd(x, 3, 2, 1)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(h_nchw(y), ry)
    a = np.transpose(arg.cpu().numpy().astype(np.int64), (0, 3, 1, 2))
    pp, qq = np.meshgrid(np.arange(p), np.arange(q), indexing="ij")
    np.testing.assert_array_equal((2 * pp + a // 3 - 1) * w + (2 * qq + a % 3 - 1), rarg)
    # the BN + ReLU in front applied as the values are loaded: same result as pooling the stored BN output
    conv = r16(synth.normal(g, shape))
    sc, sh = g.uniform(0.5, 1.5, c).astype(np.float32), synth.normal(g, c, 0.3)
    act = r16(np.maximum(np.float32(0), (conv.astype(np.float64) * sc[None, :, None, None] + sh[None, :, None, None]).astype(np.float32)))
    y2, arg2 = h_empty(n, p, q, c), torch.empty_like(arg)
    rn.maxpool3x3s2_fwd_bf16(n, c, h, w, h_nhwc(conv), to_dev(sc), to_dev(sh), y2, arg2)
    ry2, rarg2 = orc.maxpool_fwd(act, 3, 2, 1)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(h_nchw(y2), ry2)
    # backward with two incoming gradients
    dy, dy2 = r16(synth.normal(g, (n, c, p, q))), r16(synth.normal(g, (n, c, p, q)))
    dx = h_empty(n, h, w, c)
    rn.maxpool3x3s2_bwd_bf16(n, c, h, w, h_nhwc(dy), h_nhwc(dy2), arg, dx)
    torch.cuda.synchronize()
    assert_bf16(h_nchw(dx), orc.maxpool_bwd(dy.astype(np.float64) + dy2, rarg, h, w, 3, 2, 1), "maxpool bwd", frac=2e-2)
    # global average pooling: bf16 in, fp32 features; fp32 gradient in, bf16 out
    f = empty(n, c)
    rn.avgpool_fwd_bf16(n, c, h, w, h_nhwc(x), f)
    torch.cuda.synchronize()
    assert_close(f.cpu().numpy(), orc.avgpool_fwd(x), TOL, "avgpool fwd")
    df = synth.normal(g, (n, c))
    dxa = h_empty(n, h, w, c)
    rn.avgpool_bwd_bf16(n, c, h, w, to_dev(df), dxa)
    torch.cuda.synchronize()
    assert_bf16(h_nchw(dxa), orc.avgpool_bwd(df, h, w), "avgpool bwd", frac=2e-2)


# ------------------------------------------------------------------------------------------------------------------
# whole step
# ------------------------------------------------------------------------------------------------------------------
def collect_saved(ctx, batch, images_idx=None):
    """Stored forward tensors of the device run (bf16 activations widened exactly), keyed like the oracle's."""
    saved = {}
    sel = slice(None) if images_idx is None else images_idx
    for li, (name, c, k, r, stride, pad, hin) in enumerate(resnet50.conv_layers()):
        ho = orc.out_size(hin, r, stride, pad)
        saved[name + ".conv"] = nchw(ctx.peek(li, 0).view(batch, ho, ho, k)[sel])
        saved[name + ".out"] = nchw(ctx.peek(li, 1).view(batch, ho, ho, k)[sel])
        saved[name + ".mean"] = ctx.peek(li, 2).cpu().numpy().astype(np.float64)
        saved[name + ".invstd"] = ctx.peek(li, 3).cpu().numpy().astype(np.float64)
    saved["pool.out"] = nchw(ctx.peek(0, 4).view(batch, 56, 56, 64)[sel])
    a = np.transpose(ctx.peek(0, 5).view(batch, 56, 56, 64)[sel].cpu().numpy().astype(np.int64), (0, 3, 1, 2))
    pp, qq = np.meshgrid(np.arange(56), np.arange(56), indexing="ij")
    saved["pool.arg"] = ((2 * pp + a // 3 - 1) * 112 + (2 * qq + a % 3 - 1)).astype(np.int32)
    saved["feat"] = ctx.peek(0, 6).view(batch, 2048)[sel].cpu().numpy().astype(np.float64)
    saved["logits"] = ctx.peek(0, 7).view(batch, 1000)[sel].cpu().numpy().astype(np.float64)
    saved["dlogits"] = ctx.peek(0, 8).view(batch, 1000)[sel].cpu().numpy().astype(np.float64)
    return saved


class rounded_backward_ops:
    """The oracle's backward operations with a bf16 rounding at every point where the device stores an activation gradient
    (and the filter operand of the data gradient rounded as the MFMA sees it)."""

    def __enter__(self):
        self.saved = {k: getattr(orc, k) for k in ("conv2d_bwd_data", "bn_bwd", "maxpool_bwd", "avgpool_bwd")}
        o = self.saved
        orc.conv2d_bwd_data = lambda dy, w, *a: bf16_round(o["conv2d_bwd_data"](dy, bf16_round(w), *a))
        orc.maxpool_bwd = lambda dy, *a: bf16_round(o["maxpool_bwd"](dy, *a))
        orc.avgpool_bwd = lambda df, *a: bf16_round(o["avgpool_bwd"](df, *a))

        def bn_bwd(x, dy, y, gamma, mean, invstd, relu=False, want_dresidual=False):
            if want_dresidual:      # dz is stored, hence rounded, before it is used (the device sums its two gradients in fp32)
                dy = bf16_round(np.asarray(dy, dtype=np.float64).astype(np.float32))
            dx, dres, dg, db = o["bn_bwd"](x, dy, y, gamma, mean, invstd, relu=relu, want_dresidual=want_dresidual)
            return bf16_round(dx), dres, dg, db
        orc.bn_bwd = bn_bwd
        return self

    def __exit__(self, *exc):
        for k, v in self.saved.items():
            setattr(orc, k, v)


@pytest.mark.parametrize("batch", [4, 16])
def test_full_step_bf16_activations(batch):
    """Layer by layer from the device's own (bf16) inputs, every stored tensor at the one-bf16-step bar; then the oracle's
    backward on the device's forward state with a rounding wherever the device stores a gradient: close to the loss the
    two sides round identical values and agree to fp32 accuracy; further back they round values that already differ by a
    fraction of a bf16 step, so the distance grows with depth (as for any two correct bf16 evaluations) and is held to a
    bound that grows with the square root of the depth."""
    images, params, labels = problem(0, batch)
    p64 = {k: v.astype(np.float64) for k, v in params.items()}
    ctx = rn.Rn50Ctx(batch, conv_dtype=ACT)
    loss_gpu, grad, theta, dimg, dlab = gpu_forward_backward(ctx, images, params, labels, BN_EPS)
    assert math.isfinite(loss_gpu)
    saved = collect_saved(ctx, batch)
    t = dict(saved)
    t["images"] = images
    worst_frac = 0.0
    for name, src, res, relu, stride, pad in resnet50.wiring():
        conv = orc.conv2d_fwd(bf16_round(t[src]), bf16_round(p64[name + ".w"]), stride, pad)
        _, f1 = assert_bf16(saved[name + ".conv"], conv, name + " conv (device input)")
        y, mean, inv = orc.bn_fwd(saved[name + ".conv"], p64[name + ".g"], p64[name + ".beta"], BN_EPS, residual=t[res] if res else None, relu=relu)
        _, f2 = assert_bf16(saved[name + ".out"], y, name + " BN out (device input)")
        assert_close(saved[name + ".mean"], mean, TOL, name + " mean")
        assert_close(saved[name + ".invstd"], inv, TOL, name + " invstd")
        worst_frac = max(worst_frac, f1, f2)
        last = name
    py, parg = orc.maxpool_fwd(saved["stem.out"], 3, 2, 1)
    np.testing.assert_array_equal(saved["pool.out"], py)
    np.testing.assert_array_equal(saved["pool.arg"], parg)
    assert_close(saved["feat"], orc.avgpool_fwd(saved[last + ".out"]), TOL, "features")
    assert_close(saved["logits"], orc.fc_fwd(saved["feat"], p64["fc.w"], p64["fc.b"]), TOL, "logits")
    rl, rdl = orc.softmax_ce(saved["logits"], labels)
    assert abs(loss_gpu - rl) <= 1e-5 * abs(rl)
    assert_close(saved["dlogits"], rdl, TOL, "dlogits")
    ctx.close()

    g_gpu = dict_from_flat(grad.cpu().numpy())
    assert all(np.all(np.isfinite(v)) for v in g_gpu.values())
    with rounded_backward_ops():
        rg = resnet50.backward(resnet50.state_from_saved(p64, images, labels, saved), p64)
    err = {k: rel_l2(g_gpu[k], rg[k]) for k in rg}
    print("bf16 activations, N=%d: loss %.5f; forward layer by layer: at most %.1e of a tensor's elements one bf16 step off; backward on the "
          "device state with the same roundings: %s; worst %.2e (%s), median %.2e"
          % (batch, loss_gpu, worst_frac, ", ".join("%s %.1e" % (k, err[k]) for k in ("fc.w", "s5.b2.c.w", "s5.b2.b.w", "s5.b2.a.w", "s4.b0.a.w", "stem.w")),
             max(err.values()), max(err, key=err.get), float(np.median(list(err.values())))), flush=True)
    assert err["fc.w"] <= TOL and err["fc.b"] <= TOL and err["s5.b2.c.w"] <= TOL     # identical rounded values on both sides
    # Behind that the two sides round values that already differ by a fraction of a bf16 step, their rounding errors
    # (2^-9 relative, two stores per layer) become independent, and the distance between ANY two correct bf16 evaluations
    # grows like the square root of the number of layers behind the loss: measured 2.7e-3 * sqrt(depth), 1.9e-2 at the first
    # layer.  A wiring mistake would show as a jump of order one at its layer.
    names = [w_[0] for w_ in resnet50.wiring()]
    for depth, nm in enumerate(reversed(names)):
        for suffix in (".w", ".g", ".beta"):
            tol = 1e-4 + 4e-3 * math.sqrt(depth + 1)
            if nm == "stem" and suffix != ".w":
                tol = 0.12      # sums of 50,000 x N masked gradients per channel that cancel almost completely
            assert err[nm + suffix] <= tol, (nm + suffix, depth, err[nm + suffix], tol)


def test_step_bf16_activations_at_batch_256():
    """The sweep's largest batch, whole rn50_step with the measured plans.  The oracle redoes what it can at this size: every
    convolution on three sampled images of the device's own input, BN on the device's own input for layers of three sizes, the
    head; the gradients are held to properties that need no reference: finite, <W, dW> = 0 for every filter in front of a
    batch-statistics BN (up to the bf16 noise), rows of dlogits summing to zero."""
    batch = 256
    images, params, labels = problem(5, batch)
    p64 = {k: v.astype(np.float64) for k, v in params.items()}
    ctx = rn.Rn50Ctx(batch, conv_dtype=ACT)
    theta = to_dev(flat_from_dict(params))
    dimg = torch.from_numpy(np.ascontiguousarray(images.transpose(0, 2, 3, 1))).to(DEV)
    dlab = torch.from_numpy(labels).to(DEV)
    grad, delta, m = torch.empty_like(theta), torch.zeros_like(theta), torch.zeros_like(theta)
    g16 = torch.empty(theta.numel(), dtype=torch.int16, device=DEV)
    loss = empty(1)
    hp = rn.opt_hparams(0.1, 0.9, 0.99, 1e-8, 1.0, 0.0, wd=0.0, g_scale=1.0)
    ctx.step(dimg, dlab, theta, grad, delta, m, g16, hp, BN_EPS, loss)
    torch.cuda.synchronize()
    lv = loss.item()
    assert math.isfinite(lv) and abs(lv - math.log(1000.0)) < 0.5
    imgs = [0, batch // 2, batch - 1]
    saved = collect_saved(ctx, batch, imgs)
    t = dict(saved)
    t["images"] = images[imgs]
    for name, src, res, relu, stride, pad in resnet50.wiring():
        conv = orc.conv2d_fwd(bf16_round(t[src]), bf16_round(p64[name + ".w"]), stride, pad)
        assert_bf16(saved[name + ".conv"], conv, name + " conv (device input, sampled images)")
    layers = {l[0]: (i, l) for i, l in enumerate(resnet50.conv_layers())}
    for name in ("s2.b1.a", "s3.b2.c", "s5.b1.b"):
        li, (_, c, k, r, stride, pad, hin) = layers[name]
        ho = orc.out_size(hin, r, stride, pad)
        conv_full = nchw(ctx.peek(li, 0).view(batch, ho, ho, k))
        res = None
        if name.endswith(".c"):
            prev = [w_ for w_ in resnet50.wiring() if w_[0] == name][0][2]
            pli = layers[prev[:-4]][0]
            res = nchw(ctx.peek(pli, 1).view(batch, ho, ho, k))
        y, mean, inv = orc.bn_fwd(conv_full, p64[name + ".g"], p64[name + ".beta"], BN_EPS, residual=res, relu=True)
        assert_bf16(nchw(ctx.peek(li, 1).view(batch, ho, ho, k)), y, name + " BN out (device input, all images)")
        assert_close(ctx.peek(li, 2).cpu().numpy(), mean, TOL, name + " mean")
        assert_close(ctx.peek(li, 3).cpu().numpy(), inv, TOL, name + " invstd")
    assert_close(saved["logits"], orc.fc_fwd(saved["feat"], p64["fc.w"], p64["fc.b"]), TOL, "logits")
    g = grad.cpu().numpy()
    assert np.all(np.isfinite(g))
    g_gpu = dict_from_flat(g)
    for name, _, kind in resnet50.param_table():
        if kind == "conv_w":
            w_, dw = p64[name], g_gpu[name]
            assert abs(np.sum(w_ * dw)) <= 3e-2 * np.linalg.norm(w_) * np.linalg.norm(dw), name
    assert abs(g_gpu["fc.b"].sum()) <= 1e-5 * np.abs(g_gpu["fc.b"]).sum() + 1e-7
    # momentum SGD from zero state without decay: the momentum buffer is minus the gradient that went through the fp16 buffer
    np.testing.assert_array_equal(g16.cpu().numpy().view(np.uint16), orc.grad_pack_fp16(g))
    assert_close(delta.cpu().numpy(), -orc.grad_unpack_fp16(orc.grad_pack_fp16(g), 1.0), 1e-6, "delta")
    ctx.close()
