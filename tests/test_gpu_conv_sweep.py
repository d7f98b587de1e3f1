"""GPU parity of the convolutions at the batch sizes of the batch sweep (64, 128, 256), in the launch configuration the
benchmark times: every row of the measured plan table (tile shape, split factor, persistent full-tile rounds, split tail)
is launched with the shape it was measured for.

At these sizes the oracle cannot redo a whole layer, but it can compute outputs one by one: a convolution and its data
gradient are independent per image (first, middle and last image are checked, every output of each), and a filter
gradient is independent per output channel (first and last channel, summed over every image and pixel).  At batch 256
the same launches are repeated with operands rounded to bf16 on their way into LDS: there the grid is persistent and runs
whole-tile rounds with the XCD-aware tile order, which the smaller bf16 cases never reach.
"""
import os
import re

import numpy as np
import pytest
import torch

from oracle import ops as orc
from paper_1711_04325_amd import binding as rn
from paper_1711_04325_amd import synth
from tests.gpu_util import DEV, TOL, assert_close, bf16_round, empty, nhwc, ws_bytes

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def plan_rows(name="conv_plans.inc"):
    """Rows {op, n, c, h, k, r, stride, pad, bm, bn, split} of a measured plan table, from its source file."""
    txt = open(os.path.join(ROOT, "paper_1711_04325_amd", "csrc", name)).read()
    return [tuple(int(v) for v in m.group(1).split(",")) for m in re.finditer(r"^\s*\{([-0-9, ]+)\},", txt, flags=re.M)]


def shapes_at(batch):
    """Unique (n, c, h, w, k, r, stride, pad) of the table's rows at one batch size, with the directions that have a row."""
    seen = {}
    for op, n, c, h, k, r, stride, pad, bm, bn, split in plan_rows():
        if n == batch:
            seen.setdefault((n, c, h, h, k, r, stride, pad), set()).add(op)
    return sorted(seen.items())


def test_plan_table_covers_the_sweep():
    """59 rows per batch size of the sweep: 20 layer shapes x 3 directions, less the first layer's unused data gradient."""
    for batch in (64, 128, 256):
        sh = shapes_at(batch)
        assert len(sh) == 20 and sum(len(ops) for _, ops in sh) == 59
    # the table of the bf16-activation calls (its rows are launched by tests/test_gpu_bf16act.py): N=32 and N=256
    act = plan_rows("conv_plans_bf16act.inc")
    for batch in (32, 256):
        rows = [r for r in act if r[1] == batch]
        assert len(rows) == 59 and len({r[2:8] for r in rows}) == 20
        assert all(r[8] == 64 and r[9] == 64 for r in rows if r[0] == 2)   # that filter gradient has 64x64 tiles only


def _nchw_slice(t, idx):
    """Images (or filters) idx of a device NHWC tensor as logical NCHW float64."""
    return np.transpose(t[idx].detach().cpu().numpy().astype(np.float64), (0, 3, 1, 2))


SWEEP_CASES = [(case, tuple(sorted(ops))) for batch in (64, 128, 256) for case, ops in shapes_at(batch)]


@pytest.mark.gpu
@pytest.mark.parametrize("case,ops", SWEEP_CASES, ids=["n%d_c%d_h%d_k%d_r%d_s%d" % (c[0], c[1], c[2], c[4], c[5], c[6]) for c, _ in SWEEP_CASES])
def test_conv_plan_rows_on_sampled_outputs(case, ops):
    rn.rn50_set_option("igemm_plan", None)
    rn.rn50_set_option("wgrad_plan", None)
    n, c, h, w, k, r, stride, pad = case
    g = synth.rng(1000 + sum(case))
    x = synth.normal(g, (n, c, h, w))
    wt = synth.he_normal(g, (k, c, r, r))
    p, q = orc.out_size(h, r, stride, pad), orc.out_size(w, r, stride, pad)
    dy = synth.normal(g, (n, k, p, q))
    dx_, dw_, ddy_ = nhwc(x), nhwc(wt), nhwc(dy)
    imgs = [0, n // 2, n - 1]
    chans = [0, k - 1]
    # what the oracle needs, computed once: three images in both directions, two output channels of the filter gradient
    xs, dys = x[imgs], dy[imgs]
    dyc = np.ascontiguousarray(dy[:, chans])
    ref = {}
    for tag, rnd in (("f32", lambda a: a),) + ((("bf16", bf16_round),) if n == 256 else ()):
        ref[tag] = (orc.conv2d_fwd(rnd(xs), rnd(wt), stride, pad),
                    orc.conv2d_bwd_data(rnd(dys), rnd(wt), stride, pad, h, w) if 1 in ops else None,
                    orc.conv2d_bwd_weight(rnd(x), rnd(dyc), r, r, stride, pad))
    del x, dy
    for tag, in_dtype in (("f32", rn.DTYPE_F32), ("bf16", rn.DTYPE_BF16)):
        if tag not in ref:
            continue
        d = rn.conv_desc(n, c, h, w, k, r, r, stride, pad, in_dtype=in_dtype)
        y = empty(n, p, q, k)
        rn.conv2d_fwd(d, dx_, dw_, y, ws_bytes(rn.rn50_conv_workspace_bytes(d, rn.OP_FWD)))
        gdw = empty(k, r, r, c)
        rn.conv2d_bwd_weight(d, dx_, ddy_, gdw, ws_bytes(rn.rn50_conv_workspace_bytes(d, rn.OP_BWD_WEIGHT)))
        torch.cuda.synchronize()
        ry, rdx, rdw = ref[tag]
        what = "%s %s" % (tag, case)
        assert_close(_nchw_slice(y, imgs), ry, TOL, "fwd " + what)
        assert bool(torch.isfinite(y).all()), "fwd " + what
        assert_close(_nchw_slice(gdw, chans), rdw, TOL, "bwd_weight " + what)
        assert bool(torch.isfinite(gdw).all()), "bwd_weight " + what
        del y
        if 1 in ops:
            gdx = empty(n, h, w, c)
            rn.conv2d_bwd_data(d, ddy_, dw_, gdx, ws_bytes(rn.rn50_conv_workspace_bytes(d, rn.OP_BWD_DATA)))
            torch.cuda.synchronize()
            assert_close(_nchw_slice(gdx, imgs), rdx, TOL, "bwd_data " + what)
            assert bool(torch.isfinite(gdx).all()), "bwd_data " + what
            del gdx
        if tag == "bf16":   # the rounding is really there, and stays within the variant's stated tolerance of the unrounded result
            assert_close(_nchw_slice(gdw, chans), ref["f32"][2], 1e-2, "bf16 bwd_weight vs unrounded " + what)
