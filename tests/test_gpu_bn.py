"""GPU parity of batch normalization with current-minibatch statistics (forward and backward, fused residual/ReLU)."""
import numpy as np
import pytest
import torch

from oracle import ops as orc
from paper_1711_04325_amd import binding as rn
from paper_1711_04325_amd import synth
from tests.gpu_util import DEV, TOL, assert_close, empty, nchw, nhwc, to_dev, ws_bytes

pytestmark = pytest.mark.gpu

# (n, c, h, w): single band / many bands, ragged row counts, channel counts below, at and above one column block
SHAPES = [(2, 64, 56, 56), (3, 24, 5, 7), (2, 2048, 7, 7), (4, 256, 14, 14), (1, 4, 1, 3), (2, 1028, 3, 3), (32, 64, 28, 28)]


def _inputs(seed, shape, offset=2.0):
    g = synth.rng(seed)
    n, c, h, w = shape
    x = synth.normal(g, shape) * g.uniform(0.5, 2.0, size=(1, c, 1, 1)).astype(np.float32) + g.uniform(-offset, offset, size=(1, c, 1, 1)).astype(np.float32)
    gamma = synth.normal(g, c, 0.1, 1.0)
    beta = synth.normal(g, c, 0.1)
    res = synth.normal(g, shape)
    dy = synth.normal(g, shape)
    dy2 = synth.normal(g, shape)
    return x.astype(np.float32), gamma, beta, res, dy, dy2


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("relu,use_res", [(0, 0), (1, 0), (1, 1), (0, 1)])
def test_bn_fwd(shape, relu, use_res):
    n, c, h, w = shape
    x, gamma, beta, res, _, _ = _inputs(sum(shape) + relu + 2 * use_res, shape)
    eps = 2e-5
    ws = ws_bytes(rn.rn50_bn_workspace_bytes(n, c, h, w))
    y, mean, invstd = empty(n, h, w, c), empty(c), empty(c)
    rn.bn_fwd_batchstats(n, c, h, w, nhwc(x), to_dev(gamma), to_dev(beta), eps, nhwc(res) if use_res else None, relu, y, mean, invstd, ws)
    ry, rmean, rinv = orc.bn_fwd(x, gamma, beta, eps, residual=res if use_res else None, relu=bool(relu))
    assert_close(nchw(y), ry, TOL, "y")
    assert_close(mean.cpu().numpy(), rmean, TOL, "mean")
    assert_close(invstd.cpu().numpy(), rinv, TOL, "invstd")


@pytest.mark.parametrize("shape", SHAPES)
def test_bn_stats_scale_shift(shape):
    """The statistics half alone: mean, 1/sigma, and the scale and shift with which BN(x) = x*scale + shift; they are the
    very values bn_fwd_batchstats normalises with (bit-identical statistics, and its output equals fma(x, scale, shift))."""
    n, c, h, w = shape
    x, gamma, beta, _, _, _ = _inputs(5 + sum(shape), shape)
    eps = 2e-5
    ws = ws_bytes(rn.rn50_bn_workspace_bytes(n, c, h, w))
    mean, invstd, scale, shift = empty(c), empty(c), empty(c), empty(c)
    rn.bn_stats_scale_shift(n, c, h, w, nhwc(x), to_dev(gamma), to_dev(beta), eps, mean, invstd, scale, shift, ws)
    _, rmean, rinv = orc.bn_fwd(x, gamma, beta, eps)
    assert_close(mean.cpu().numpy(), rmean, TOL, "mean")
    assert_close(invstd.cpu().numpy(), rinv, TOL, "invstd")
    assert_close(scale.cpu().numpy(), gamma.astype(np.float64) * rinv, TOL, "scale")
    assert_close(shift.cpu().numpy(), beta.astype(np.float64) - rmean * gamma.astype(np.float64) * rinv, TOL, "shift")
    y, mean2, invstd2 = empty(n, h, w, c), empty(c), empty(c)
    rn.bn_fwd_batchstats(n, c, h, w, nhwc(x), to_dev(gamma), to_dev(beta), eps, None, 0, y, mean2, invstd2, ws)
    np.testing.assert_array_equal(mean.cpu().numpy().view(np.uint32), mean2.cpu().numpy().view(np.uint32))
    np.testing.assert_array_equal(invstd.cpu().numpy().view(np.uint32), invstd2.cpu().numpy().view(np.uint32))
    want = torch.addcmul(shift.double(), nhwc(x).double(), scale.double()).float()   # one rounding, as fmaf
    np.testing.assert_array_equal(y.cpu().numpy().view(np.uint32), want.cpu().numpy().view(np.uint32))


def test_bn_fwd_large_mean_is_stable():
    # |mean| >> std: a sum / sum-of-squares formulation would lose the variance
    shape = (8, 32, 16, 16)
    n, c, h, w = shape
    g = synth.rng(3)
    x = (synth.normal(g, shape, 0.01) + np.float32(100.0)).astype(np.float32)
    gamma, beta = np.ones(c, np.float32), np.zeros(c, np.float32)
    ws = ws_bytes(rn.rn50_bn_workspace_bytes(n, c, h, w))
    y, mean, invstd = empty(n, h, w, c), empty(c), empty(c)
    rn.bn_fwd_batchstats(n, c, h, w, nhwc(x), to_dev(gamma), to_dev(beta), 1e-10, None, 0, y, mean, invstd, ws)
    ry, rmean, rinv = orc.bn_fwd(x, gamma, beta, 1e-10)
    assert_close(invstd.cpu().numpy(), rinv, 1e-4, "invstd")
    assert_close(mean.cpu().numpy(), rmean, 1e-6, "mean")


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("relu,use_res,use_dy2", [(0, 0, 0), (1, 0, 0), (1, 1, 1), (1, 1, 0), (1, 0, 1), (0, 1, 0), (0, 0, 1)])
def test_bn_bwd(shape, relu, use_res, use_dy2):
    n, c, h, w = shape
    x, gamma, beta, res, dy, dy2 = _inputs(7 + sum(shape) + relu + 2 * use_res + 4 * use_dy2, shape, offset=1.0)
    eps = 2e-5
    # identical fp32 inputs on both sides, including the saved forward tensors (produced by the oracle, rounded to
    # fp32): the ReLU mask is then a function of the inputs only
    ry, rmean, rinv = orc.bn_fwd(x, gamma, beta, eps, residual=res if use_res else None, relu=bool(relu))
    y32, mean32, inv32 = ry.astype(np.float32), rmean.astype(np.float32), rinv.astype(np.float32)
    dy_tot = dy.astype(np.float64) + (dy2.astype(np.float64) if use_dy2 else 0.0)
    rdx, rdres, rdg, rdb = orc.bn_bwd(x, dy_tot, y32, gamma, mean32, inv32, relu=bool(relu), want_dresidual=bool(use_res))
    ws = ws_bytes(rn.rn50_bn_workspace_bytes(n, c, h, w))
    dx, dres, dg, db = empty(n, h, w, c), (empty(n, h, w, c) if use_res else None), empty(c), empty(c)
    rn.bn_bwd_batchstats(n, c, h, w, nhwc(x), nhwc(dy), nhwc(dy2) if use_dy2 else None, nhwc(y32) if relu else None, to_dev(gamma),
                         to_dev(mean32), to_dev(inv32), relu, dx, dres, dg, db, ws)
    assert_close(nchw(dx), rdx, TOL, "dx")
    assert_close(dg.cpu().numpy(), rdg, TOL, "dgamma")
    assert_close(db.cpu().numpy(), rdb, TOL, "dbeta")
    if use_res:
        assert_close(nchw(dres), rdres, TOL, "dresidual")


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("use_res,use_dy2", [(1, 1), (0, 0), (1, 0)])
def test_bn_relu_byte_mask(shape, use_res, use_dy2):
    """bn_fwd_batchstats_mask writes one byte per four channels with bit e = [y > 0]; bn_bwd_batchstats_mask reads it instead
    of y: the mask equals the oracle's [y > 0] wherever the oracle's pre-activation is not within rounding of zero, the
    forward output is that of bn_fwd_batchstats bit for bit, and the backward pass gives the same bits as the y-reading one."""
    n, c, h, w = shape
    x, gamma, beta, res, dy, dy2 = _inputs(23 + sum(shape) + use_res + 2 * use_dy2, shape, offset=1.0)
    eps = 2e-5
    ws = ws_bytes(rn.rn50_bn_workspace_bytes(n, c, h, w))
    dx_, dg_, db_, dres_ = nhwc(x), to_dev(gamma), to_dev(beta), (nhwc(res) if use_res else None)
    y, mean, invstd = empty(n, h, w, c), empty(c), empty(c)
    mask = torch.full((n * h * w * c // 4,), 0xFF, dtype=torch.uint8, device=DEV)
    rn.bn_fwd_batchstats_mask(n, c, h, w, dx_, dg_, db_, eps, dres_, y, mask, mean, invstd, ws)
    y2, mean2, invstd2 = empty(n, h, w, c), empty(c), empty(c)
    rn.bn_fwd_batchstats(n, c, h, w, dx_, dg_, db_, eps, dres_, 1, y2, mean2, invstd2, ws)
    np.testing.assert_array_equal(y.cpu().numpy().view(np.uint32), y2.cpu().numpy().view(np.uint32))
    bits = np.unpackbits(mask.cpu().numpy()[:, None], axis=1, bitorder="little")[:, :4].reshape(n, h, w, c)
    np.testing.assert_array_equal(bits.astype(bool), y.cpu().numpy() > 0)
    assert int(mask.max().item()) < 16
    ry, _, _ = orc.bn_fwd(x, gamma, beta, eps, residual=res if use_res else None, relu=False)
    sure = np.abs(ry) > 1e-5   # away from the ReLU kink the fp32 and fp64 signs agree
    np.testing.assert_array_equal(np.transpose(bits, (0, 3, 1, 2)).astype(bool)[sure], (ry > 0)[sure])
    outs = []
    for use_mask in (True, False):
        dx, dres, dg, db = empty(n, h, w, c), (empty(n, h, w, c) if use_res else None), empty(c), empty(c)
        if use_mask:
            rn.bn_bwd_batchstats_mask(n, c, h, w, dx_, nhwc(dy), nhwc(dy2) if use_dy2 else None, mask, dg_, mean, invstd, dx, dres, dg, db, ws)
        else:
            rn.bn_bwd_batchstats(n, c, h, w, dx_, nhwc(dy), nhwc(dy2) if use_dy2 else None, y, dg_, mean, invstd, 1, dx, dres, dg, db, ws)
        outs.append([t.cpu().numpy().view(np.uint32).copy() for t in (dx, dg, db) + ((dres,) if use_res else ())])
    for a, b in zip(*outs):
        np.testing.assert_array_equal(a, b)


def test_bn_is_deterministic():
    shape = (8, 128, 28, 28)
    n, c, h, w = shape
    x, gamma, beta, res, dy, _ = _inputs(1, shape)
    ws = ws_bytes(rn.rn50_bn_workspace_bytes(n, c, h, w))
    outs = []
    dx_, dg_, db_ = nhwc(x), to_dev(gamma), to_dev(beta)
    for _ in range(2):
        y, mean, invstd = empty(n, h, w, c), empty(c), empty(c)
        rn.bn_fwd_batchstats(n, c, h, w, dx_, dg_, db_, 2e-5, None, 1, y, mean, invstd, ws)
        outs.append((y.cpu().numpy().copy(), mean.cpu().numpy().copy(), invstd.cpu().numpy().copy()))
    for a, b in zip(*outs):
        np.testing.assert_array_equal(a.view(np.uint32), b.view(np.uint32))


def test_bn_workspace_reused_across_calls_with_other_data_and_shapes():
    """One workspace serves calls of different shapes and data back to back (as inside a training step): no call may
    read partial sums that an earlier one left there."""
    shapes = [(8, 128, 28, 28), (4, 256, 14, 14), (8, 128, 28, 28), (2, 2048, 7, 7), (32, 64, 28, 28), (8, 128, 28, 28)]
    ws = ws_bytes(max(rn.rn50_bn_workspace_bytes(*s) for s in shapes))
    eps = 2e-5
    pending = []
    for i, shape in enumerate(shapes):   # all calls enqueued before any result is read back
        n, c, h, w = shape
        x, gamma, beta, _, dy, _ = _inputs(100 + i, shape, offset=1.0)
        y, mean, invstd = empty(n, h, w, c), empty(c), empty(c)
        rn.bn_fwd_batchstats(n, c, h, w, nhwc(x), to_dev(gamma), to_dev(beta), eps, None, 1, y, mean, invstd, ws)
        ry, rmean, rinv = orc.bn_fwd(x, gamma, beta, eps, relu=True)
        y32, mean32, inv32 = ry.astype(np.float32), rmean.astype(np.float32), rinv.astype(np.float32)
        dx, dg, db = empty(n, h, w, c), empty(c), empty(c)
        rn.bn_bwd_batchstats(n, c, h, w, nhwc(x), nhwc(dy), None, nhwc(y32), to_dev(gamma), to_dev(mean32), to_dev(inv32), 1, dx, None,
                             dg, db, ws)
        rdx, _, rdg, rdb = orc.bn_bwd(x, dy, y32, gamma, mean32, inv32, relu=True)
        pending.append((y, ry, mean, rmean, dx, rdx, dg, rdg, db, rdb))
    for y, ry, mean, rmean, dx, rdx, dg, rdg, db, rdb in pending:
        assert_close(nchw(y), ry, TOL, "y")
        assert_close(mean.cpu().numpy(), rmean, TOL, "mean")
        assert_close(nchw(dx), rdx, TOL, "dx")
        assert_close(dg.cpu().numpy(), rdg, TOL, "dgamma")
        assert_close(db.cpu().numpy(), rdb, TOL, "dbeta")


def test_bn_argument_errors():
    t = empty(64)
    ws = ws_bytes(1024)
    with pytest.raises(rn.Rn50Error) as e:
        rn.bn_fwd_batchstats(1, 6, 2, 2, t, t, t, 1e-5, None, 0, t, t, t, ws)
    assert e.value.code == rn.EUNSUPPORTED
    with pytest.raises(rn.Rn50Error) as e:
        rn.bn_fwd_batchstats(1, 8, 2, 2, t, t, t, 1e-5, None, 0, t, t, t, ws, layout=rn.LAYOUT_NCHW)
    assert e.value.code == rn.EUNSUPPORTED
    with pytest.raises(rn.Rn50Error) as e:
        rn.bn_fwd_batchstats(64, 64, 56, 56, t, t, t, 1e-5, None, 0, t, t, t, ws_bytes(16))
    assert e.value.code == rn.EWORKSPACE
    with pytest.raises(rn.Rn50Error) as e:
        rn.bn_bwd_batchstats(1, 8, 2, 2, t, t, None, None, t, t, t, 1, t, None, t, t, ws)
    assert e.value.code == rn.EINVAL


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("relu,use_res", [(0, 0), (1, 0), (1, 1)])
def test_bn_fwd_inference(shape, relu, use_res):
    """Validation-side BN: given statistics (here: arbitrary ones, not the batch's)."""
    n, c, h, w = shape
    x, gamma, beta, res, _, _ = _inputs(11 + sum(shape) + relu + 2 * use_res, shape)
    g = synth.rng(5)
    mean = synth.normal(g, c)
    invstd = g.uniform(0.5, 2.0, c).astype(np.float32)
    ws = ws_bytes(rn.rn50_bn_workspace_bytes(n, c, h, w))
    y = empty(n, h, w, c)
    rn.bn_fwd_inference(n, c, h, w, nhwc(x), to_dev(gamma), to_dev(beta), to_dev(mean), to_dev(invstd),
                        nhwc(res) if use_res else None, relu, y, ws)
    assert_close(nchw(y), orc.bn_inference(x, gamma, beta, mean, invstd, residual=res if use_res else None, relu=bool(relu)), TOL, "y")


def test_bn_inference_with_the_batch_statistics_is_the_training_forward():
    shape = (4, 256, 14, 14)
    n, c, h, w = shape
    x, gamma, beta, res, _, _ = _inputs(77, shape)
    ws = ws_bytes(rn.rn50_bn_workspace_bytes(n, c, h, w))
    y, y2, mean, invstd = empty(n, h, w, c), empty(n, h, w, c), empty(c), empty(c)
    dx, dg, db, dr = nhwc(x), to_dev(gamma), to_dev(beta), nhwc(res)
    rn.bn_fwd_batchstats(n, c, h, w, dx, dg, db, 2e-5, dr, 1, y, mean, invstd, ws)
    rn.bn_fwd_inference(n, c, h, w, dx, dg, db, mean, invstd, dr, 1, y2, ws)
    np.testing.assert_array_equal(y.cpu().numpy(), y2.cpu().numpy())   # same scale/shift expressions, same apply kernel


@pytest.mark.parametrize("n_sets", [1, 2, 5])
def test_bn_stats_average(n_sets):
    c, eps = 260, 2e-5
    g = synth.rng(n_sets)
    means = synth.normal(g, (n_sets, c))
    inv = (1.0 / np.sqrt(g.uniform(0.1, 3.0, (n_sets, c)) + eps)).astype(np.float32)
    mo, io = empty(c), empty(c)
    rn.bn_stats_average(c, n_sets, to_dev(means), to_dev(inv), eps, mo, io)
    rm, ri = orc.bn_stats_average(means, inv, eps)
    assert_close(mo.cpu().numpy(), rm, TOL, "mean")
    assert_close(io.cpu().numpy(), ri, TOL, "invstd")
    if n_sets == 1:
        np.testing.assert_array_equal(mo.cpu().numpy(), means[0])


@pytest.mark.parametrize("shape", SHAPES)
def test_bn_bwd_mask_rebuilt_from_x(shape):
    """BN -> ReLU backward without the forward output: the device's own forward decides the mask on both sides, so the
    result must be BIT-identical to bn_bwd_batchstats fed with that forward output, and within the bar of the oracle."""
    n, c, h, w = shape
    x, gamma, beta, _, dy, _ = _inputs(31 + sum(shape), shape, offset=0.5)
    eps = 2e-5
    ws = ws_bytes(rn.rn50_bn_workspace_bytes(n, c, h, w))
    dxx, dg_, db_ = nhwc(x), to_dev(gamma), to_dev(beta)
    y, mean, invstd = empty(n, h, w, c), empty(c), empty(c)
    rn.bn_fwd_batchstats(n, c, h, w, dxx, dg_, db_, eps, None, 1, y, mean, invstd, ws)
    ddy = nhwc(dy)
    out = []
    for use_x in (False, True):
        dx, dgam, dbet = empty(n, h, w, c), empty(c), empty(c)
        if use_x:
            rn.bn_bwd_batchstats_xmask(n, c, h, w, dxx, ddy, dg_, db_, mean, invstd, dx, dgam, dbet, ws)
        else:
            rn.bn_bwd_batchstats(n, c, h, w, dxx, ddy, None, y, dg_, mean, invstd, 1, dx, None, dgam, dbet, ws)
        out.append((dx.cpu().numpy(), dgam.cpu().numpy(), dbet.cpu().numpy()))
    for u, v in zip(*out):
        np.testing.assert_array_equal(u.view(np.uint32), v.view(np.uint32))
    rdx, _, rdg, rdb = orc.bn_bwd(x, dy, nchw(y), gamma, mean.cpu().numpy().astype(np.float64), invstd.cpu().numpy().astype(np.float64), relu=True)
    assert_close(nchw(torch.from_numpy(out[1][0])), rdx, TOL, "dx")
    assert_close(out[1][1], rdg, TOL, "dgamma")
    assert_close(out[1][2], rdb, TOL, "dbeta")


# The benchmarked tensors (a stage-2 block output and the stem's output at N = 32) and the a/b-layer tensor of stage 2 at the
# largest batch of the sweep: here the reductions run with their maximum of 512 row bands and the element-wise passes with
# their own finer cut, which the small shapes above never reach.  The oracle still does the whole tensor.
FULL_SHAPES = [(32, 256, 56, 56), (32, 64, 112, 112), (256, 64, 56, 56)]


@pytest.mark.parametrize("shape", FULL_SHAPES)
def test_bn_at_full_size(shape):
    test_bn_fwd(shape, 1, 1)
    test_bn_bwd(shape, 1, 1, 1)
    test_bn_relu_byte_mask(shape, 1, 1)
    test_bn_bwd_mask_rebuilt_from_x(shape)
