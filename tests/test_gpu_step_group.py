"""Whole step with the filter gradients in grouped launches (option wgrad_group: per block, per stage, whole network):
against the layer-by-layer schedule the loss and every gradient that is not a convolution filter's are bit-identical, the
filter gradients the same sums in another order (rel-L2 <= 1e-5 per tensor), with and without the helper streams, call
after call."""
import numpy as np
import pytest
import torch

from oracle import resnet50
from paper_1711_04325_amd import binding as rn
from tests.step_util import gpu_forward_backward, problem

pytestmark = pytest.mark.gpu
BN_EPS = 2e-5


def _run(batch, images, params, labels, group, side, variant=0, stages=None, calls=2):
    rn.rn50_set_option("wgrad_group", group)
    rn.rn50_set_option("side_stream", side)
    rn.rn50_set_option("wgrad_group_stages", stages)
    try:
        ctx = rn.Rn50Ctx(batch, variant=variant)
    finally:
        rn.rn50_set_option("wgrad_group", None)
        rn.rn50_set_option("side_stream", None)
        rn.rn50_set_option("wgrad_group_stages", None)
    outs = []
    for _ in range(calls):
        loss, grad, *_ = gpu_forward_backward(ctx, images, params, labels, BN_EPS)
        outs.append((np.float32(loss), grad.cpu().numpy().copy()))
    ctx.close()
    for loss, g in outs[1:]:
        assert loss == outs[0][0]
        np.testing.assert_array_equal(g.view(np.uint32), outs[0][1].view(np.uint32))
    return outs[0]


@pytest.mark.parametrize("variant", [0, 1])
def test_grouped_filter_gradients_match_the_layerwise_schedule(variant):
    batch = 4
    images, params, labels = problem(21, batch)
    loss0, g0 = _run(batch, images, params, labels, "0", "1", variant)
    table = rn.rn50_param_table()
    for group in ("1", "3", "16"):
        per_side = []
        for side in ("1", "0"):
            loss, g = _run(batch, images, params, labels, group, side, variant)
            assert loss == loss0
            per_side.append(g)
            for name, off, cnt, dims, kind in table:
                a, b = g[off:off + cnt], g0[off:off + cnt]
                if kind == 0 and name != "stem.w":
                    err = np.linalg.norm(a.astype(np.float64) - b) / np.linalg.norm(b.astype(np.float64))
                    assert err <= 1e-5, (group, side, name, err)
                else:   # BN and FC gradients and the first layer's filter gradient come from the same kernels as before
                    np.testing.assert_array_equal(a.view(np.uint32), b.view(np.uint32), err_msg=name)
        np.testing.assert_array_equal(per_side[0].view(np.uint32), per_side[1].view(np.uint32))


def test_grouped_filter_gradients_with_short_work_items():
    """Work items shorter than the workspace was planned for are not accepted: the context falls back to the planned minimum
    (16 stages), and longer ones cut the pixels differently; both give the same gradients."""
    batch = 3
    images, params, labels = problem(22, batch)
    loss0, g0 = _run(batch, images, params, labels, "0", "1", calls=1)
    for stages in ("2", "100"):
        loss, g = _run(batch, images, params, labels, "1", "1", stages=stages, calls=1)
        assert loss == loss0
        for name, off, cnt, dims, kind in rn.rn50_param_table():
            a, b = g[off:off + cnt].astype(np.float64), g0[off:off + cnt].astype(np.float64)
            assert np.linalg.norm(a - b) <= 1e-5 * np.linalg.norm(b), (stages, name)


def test_groups_run_alone():
    """rn50_wgrad_groups_run repeats the step's grouped launches on the buffers the step left: the same gradients again."""
    batch = 2
    images, params, labels = problem(23, batch)
    rn.rn50_set_option("wgrad_group", "1")
    try:
        ctx = rn.Rn50Ctx(batch)
    finally:
        rn.rn50_set_option("wgrad_group", None)
    loss, grad, *_ = gpu_forward_backward(ctx, images, params, labels, BN_EPS)
    again = torch.full_like(grad, float("nan"))
    assert ctx.wgrad_groups_run(again) == 16
    torch.cuda.synchronize()
    for name, off, cnt, dims, kind in rn.rn50_param_table():
        if kind == 0 and name != "stem.w":
            assert torch.equal(again[off:off + cnt], grad[off:off + cnt]), name
    ctx.close()
