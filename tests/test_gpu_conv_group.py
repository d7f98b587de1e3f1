"""GPU parity of conv2d_bwd_weight_group (the filter gradients of several layers in one launch) against the fp64 oracle
(rel-L2 <= 1e-4 per layer), against conv2d_bwd_weight per layer, for every tile shape and several work-item lengths, with
ragged tiles, a fused BN + ReLU input and gradients at scattered offsets of one arena."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import ops as orc
from paper_1711_04325_amd import binding as rn
from paper_1711_04325_amd import synth
from tests.gpu_util import DEV, TOL, assert_close, empty, nchw, nhwc, rel_l2, to_dev, ws_bytes

pytestmark = pytest.mark.gpu

# (n, c, h, w, k, r, stride, pad, fused BN + ReLU input)
LAYERS = [
    (2, 64, 28, 28, 64, 3, 1, 1, False),
    (2, 64, 56, 56, 256, 1, 1, 0, True),
    (3, 256, 14, 14, 64, 1, 1, 0, False),   # 588 pixels: ragged last stage
    (2, 128, 28, 28, 96, 1, 2, 0, False),   # stride 2, K not a multiple of 64
    (1, 32, 9, 11, 40, 3, 1, 1, True),      # odd sizes, tiles ragged on both sides
    (2, 512, 7, 7, 512, 3, 1, 1, False),    # 98 pixels: a single range per tile
    (2, 64, 15, 15, 64, 3, 2, 1, False),
    (1, 20, 8, 8, 24, 3, 1, 1, False),      # one ragged tile, two stages
]


def _options(stages, tile):
    rn.rn50_set_option("wgrad_group_stages", stages)
    rn.rn50_set_option("wgrad_group_tile", tile)


def _make(layers, seed):
    g = synth.rng(seed)
    host, dev, off = [], [], 0
    for (n, c, h, w, k, r, stride, pad, fused) in layers:
        x = synth.normal(g, (n, c, h, w))
        p, q = orc.out_size(h, r, stride, pad), orc.out_size(w, r, stride, pad)
        dy = synth.normal(g, (n, k, p, q))
        sc = sh = None
        if fused:
            sc = 1.0 + 0.1 * synth.normal(g, (c,))
            sh = 0.1 * synth.normal(g, (c,))
        off = (off + 63) // 64 * 64 + 64  # a gap before every gradient: nothing may be written there
        host.append((x, dy, sc, sh, off))
        d = rn.conv_desc(n, c, h, w, k, r, r, stride, pad)
        dev.append((d, nhwc(x), None if sc is None else to_dev(sc), None if sh is None else to_dev(sh), nhwc(dy), off))
        off += k * r * r * c
    return host, dev, off + 64


def _run_group(dev, total):
    items = rn.wgrad_group_items(dev)
    ws = ws_bytes(rn.rn50_wgrad_group_workspace_bytes(items))
    table = rn.rn50_wgrad_group_plan(items, ws)
    table_dev = torch.frombuffer(bytearray(table.raw), dtype=torch.uint8).to(DEV)
    arena = torch.full((total,), float("nan"), dtype=torch.float32, device=DEV)
    rn.conv2d_bwd_weight_group(table, table_dev, arena)
    torch.cuda.synchronize()
    return arena, (table, table_dev, ws)


def _check(layers, seed):
    host, dev, total = _make(layers, seed)
    arena, keep = _run_group(dev, total)
    a = arena.cpu().numpy()
    written = np.zeros(total, dtype=bool)
    for (n, c, h, w, k, r, stride, pad, fused), (x, dy, sc, sh, off), (d, dx_, dsc, dsh, ddy_, _) in zip(layers, host, dev):
        cnt = k * r * r * c
        got = np.transpose(a[off:off + cnt].astype(np.float64).reshape(k, r, r, c), (0, 3, 1, 2))
        xin = x if sc is None else np.maximum(x.astype(np.float64) * np.float32(sc).astype(np.float64)[None, :, None, None]
                                              + np.float32(sh).astype(np.float64)[None, :, None, None], 0.0)
        assert_close(got, orc.conv2d_bwd_weight(xin, dy, r, r, stride, pad), TOL, "group bwd_weight %s" % ((n, c, h, w, k, r, stride, pad),))
        # the per-layer call on the same device tensors: same sums in another order
        one = empty(k, r, r, c)
        wsb = ws_bytes(rn.rn50_conv_workspace_bytes(d, rn.OP_BWD_WEIGHT))
        if sc is None:
            rn.conv2d_bwd_weight(d, dx_, ddy_, one, wsb)
        else:
            rn.conv2d_bwd_weight_bnrelu_input(d, dx_, dsc, dsh, ddy_, one, wsb)
        torch.cuda.synchronize()
        assert rel_l2(got, nchw(one)) <= 1e-5
        written[off:off + cnt] = True
    assert np.all(np.isfinite(a[written])) and np.all(np.isnan(a[~written])), "something outside the gradients was written"
    # bit-identical from launch to launch
    again = torch.full_like(arena, float("nan"))
    rn.conv2d_bwd_weight_group(keep[0], keep[1], again)
    torch.cuda.synchronize()
    assert torch.equal(arena[torch.from_numpy(written).to(DEV)], again[torch.from_numpy(written).to(DEV)])


@pytest.mark.parametrize("tile", ["64,64", "128,64", "64,128", "128,128"])
@pytest.mark.parametrize("stages", ["2", "5", "32"])
def test_group_every_tile_and_item_length(tile, stages):
    _options(stages, tile)
    try:
        _check(LAYERS, 31)
    finally:
        _options(None, None)


def test_group_of_one_layer_and_default_options():
    _options(None, None)
    for i, layer in enumerate(LAYERS[:3]):
        _check([layer], 40 + i)


def test_group_rejects_bad_arguments():
    d = rn.conv_desc(2, 64, 8, 8, 64, 3, 3, 1, 1)
    x, dy = empty(2, 8, 8, 64), empty(2, 8, 8, 64)
    items = rn.wgrad_group_items([(d, x, None, None, dy, 0)])
    ws = ws_bytes(rn.rn50_wgrad_group_workspace_bytes(items))
    with pytest.raises(rn.Rn50Error):  # workspace too small
        rn.rn50_wgrad_group_plan(items, ws[:64])
    with pytest.raises(rn.Rn50Error):  # gradient offset not a multiple of 4
        rn.rn50_wgrad_group_plan(rn.wgrad_group_items([(d, x, None, None, dy, 2)]), ws)
    with pytest.raises(rn.Rn50Error):  # scale without shift
        rn.rn50_wgrad_group_plan(rn.wgrad_group_items([(d, x, x, None, dy, 0)]), ws)
    d3 = rn.conv_desc(2, 3, 8, 8, 64, 3, 3, 1, 1)
    assert rn.rn50_wgrad_group_workspace_bytes(rn.wgrad_group_items([(d3, x, None, None, dy, 0)])) == 0  # C % 4 != 0
    table = rn.rn50_wgrad_group_plan(items, ws)
    junk = C.create_string_buffer(len(table))
    with pytest.raises(rn.Rn50Error):  # not a plan
        rn.conv2d_bwd_weight_group(junk, ws, empty(64 * 9 * 64))
