"""bn_fwd_batchstats_static, the BN forward for callers that cannot allocate: its band partials live in a buffer built
into the library instead of a caller's workspace.  Through the C ABI its outputs must equal bn_fwd_batchstats' bit for bit
(same kernels) and meet the oracle's bar, on two calls in a row, the second with a smaller input (the buffer then still
holds the first call's partials)."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import ops as orc
from paper_1711_04325_amd import binding as rn
from paper_1711_04325_amd import synth
from tests.gpu_util import DEV, TOL, assert_close, empty, nchw, nhwc, to_dev, ws_bytes


def _both(n, c, h, w, seed, with_residual, relu):
    g = synth.rng(seed)
    x = synth.normal(g, (n, c, h, w), 1.5, 0.7)
    res = synth.normal(g, (n, c, h, w)) if with_residual else None
    gamma, beta = synth.normal(g, c, 0.1, 1.0), synth.normal(g, c, 0.1)
    dx_, dres = nhwc(x), (nhwc(res) if with_residual else None)
    dga, dbe = to_dev(gamma), to_dev(beta)
    outs = []
    for static in (True, False):
        y, mean, inv = torch.full((n, h, w, c), float("nan"), device=DEV), empty(c), empty(c)
        if static:
            rn.bn_fwd_batchstats_static(n, c, h, w, dx_, dga, dbe, 2e-5, dres, relu, y, mean, inv)
        else:
            rn.bn_fwd_batchstats(n, c, h, w, dx_, dga, dbe, 2e-5, dres, relu, y, mean, inv, ws_bytes(rn.rn50_bn_workspace_bytes(n, c, h, w)))
        torch.cuda.synchronize()
        outs.append((y.cpu().numpy(), mean.cpu().numpy(), inv.cpu().numpy()))
    for a, b in zip(*outs):
        np.testing.assert_array_equal(a.view(np.uint32), b.view(np.uint32))
    ry, rmean, rinv = orc.bn_fwd(x, gamma, beta, 2e-5, residual=res, relu=bool(relu))
    assert_close(np.transpose(outs[0][0].astype(np.float64), (0, 3, 1, 2)), ry, TOL, "y")
    assert_close(outs[0][1], rmean, TOL, "mean")
    assert_close(outs[0][2], rinv, TOL, "invstd")


@pytest.mark.gpu
def test_static_scratch_bn_two_calls_in_a_row():
    _both(4, 256, 28, 28, 71, True, 1)      # 3136 rows x 256 channels: many bands
    _both(2, 64, 7, 9, 72, False, 1)        # smaller: fewer bands and channels than the partials left in the buffer
    _both(3, 2048, 7, 7, 73, False, 0)      # the widest BN of the network


def test_static_scratch_bn_rejects_what_does_not_fit():
    """Validated before any HIP call: a shape whose partials exceed the built-in buffer is refused with a clear message."""
    L = rn.lib()
    n, c, h, w = 32, 4096, 56, 56
    assert rn.rn50_bn_workspace_bytes(n, c, h, w) > rn.BN_STATIC_SCRATCH_BYTES
    assert L.bn_fwd_batchstats_static(n, c, h, w, rn.LAYOUT_NHWC, 16, 16, 16, 2e-5, None, 1, 16, 16, 16, None) == rn.EWORKSPACE
    assert b"built-in buffer" in L.rn50_last_error()
    assert L.bn_fwd_batchstats_static(2, 64, 4, 4, rn.LAYOUT_NHWC, None, 16, 16, 2e-5, None, 1, 16, 16, 16, None) == rn.EINVAL
    assert L.bn_fwd_batchstats_static(2, 6, 4, 4, rn.LAYOUT_NHWC, 16, 16, 16, 2e-5, None, 1, 16, 16, 16, None) == rn.EUNSUPPORTED
    # every BN shape of the network, at every batch size of the sweep, fits
    for batch in (1, 32, 64, 128, 256):
        for cc, hh in ((64, 112), (64, 56), (256, 56), (128, 28), (512, 28), (256, 14), (1024, 14), (512, 7), (2048, 7), (128, 56), (256, 28), (512, 14)):
            assert 0 < rn.rn50_bn_workspace_bytes(batch, cc, hh, hh) <= rn.BN_STATIC_SCRATCH_BYTES
