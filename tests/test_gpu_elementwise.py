"""GPU parity: half-precision communication buffer (bit-exact) and the update rule (rel-L2 <= 1e-4)."""
import os

import numpy as np
import pytest
import torch

from oracle import ops as orc
from paper_1711_04325_amd import binding as rn
from paper_1711_04325_amd import synth
from tests.gpu_util import DEV, TOL, assert_close, empty, to_dev

pytestmark = pytest.mark.gpu


def _pack(f):
    g = torch.from_numpy(f).to(DEV)
    out = torch.empty(f.size, dtype=torch.int16, device=DEV)
    rn.grad_pack_fp16(f.size, g, out)
    torch.cuda.synchronize()
    return out.cpu().numpy().view(np.uint16)


def _check_pack(f):
    got, ref = _pack(f), orc.grad_pack_fp16(f)
    ok = ~np.isnan(f)
    np.testing.assert_array_equal(got[ok], ref[ok])
    nan = got[~ok]
    assert np.all((nan & 0x7c00) == 0x7c00) and np.all((nan & 0x3ff) != 0)  # NaN stays NaN; payload not compared


def test_pack_boundaries_and_all_halfs(golden_dir):
    rows = [l.split("#")[0].split() for l in open(os.path.join(golden_dir, "fp16_boundaries.txt"))]
    rows = [(int(r[0], 16), int(r[1], 16)) for r in rows if len(r) == 2]
    f = np.array([r[0] for r in rows], dtype=np.uint32).view(np.float32)
    np.testing.assert_array_equal(_pack(f), np.array([r[1] for r in rows], dtype=np.uint16))
    h = np.arange(65536, dtype=np.uint16)
    f = h.view(np.float16).astype(np.float32)
    ok = ~np.isnan(f)
    np.testing.assert_array_equal(_pack(f)[ok], h[ok])
    lo = np.arange(0, 0x7bff, dtype=np.uint16)
    mid = ((lo.view(np.float16).astype(np.float64) + (lo + 1).astype(np.uint16).view(np.float16).astype(np.float64)) / 2).astype(np.float32)
    for arr in (mid, -mid, np.nextafter(mid, np.float32(np.inf)), np.nextafter(mid, np.float32(-np.inf))):
        _check_pack(arr)


@pytest.mark.parametrize("count", [1, 7, 8, 9, 1000, 2047, 262144 + 5, 3_000_001])
def test_pack_random_bits_ragged(count):
    g = synth.rng(count)
    _check_pack(synth.fp32_bit_patterns(g, count))
    _check_pack(synth.gradient_like(g, count))


def test_pack_full_arena_size():
    n = rn.rn50_param_count()
    assert n == 25_557_032
    g = synth.rng(11)
    _check_pack(synth.gradient_like(g, n))
    _check_pack(synth.fp32_bit_patterns(g, n))


def test_pack_empty():
    rn.grad_pack_fp16(0, 0, 0)
    rn.grad_unpack_fp16(0, 0, 1.0, 0)


@pytest.mark.parametrize("count", [5, 65536, 1_000_003])
def test_unpack_bit_exact(count):
    g = synth.rng(count)
    h = g.integers(0, 65536, size=count, dtype=np.uint16) if count != 65536 else np.arange(65536, dtype=np.uint16)
    d = torch.from_numpy(h.view(np.int16)).to(DEV)
    out = empty(count)
    for scale in (1.0, 1.0 / 1024):
        rn.grad_unpack_fp16(count, d, scale, out)
        got = out.cpu().numpy()
        ref = orc.grad_unpack_fp16(h, scale).astype(np.float32)  # exact: power-of-two scale
        ok = ~np.isnan(ref)
        np.testing.assert_array_equal(got[ok].view(np.uint32), ref[ok].view(np.uint32))
        assert np.all(np.isnan(got[~ok]))


BLENDS = [0.0, 5.0, 10.0, 11.25, 12.5]  # epochs: alpha_SGD = 0.0092, 0.068, 0.5, 0.75, 1


@pytest.mark.parametrize("epoch", BLENDS)
@pytest.mark.parametrize("use_half", [False, True])
def test_opt_update_blend_points(epoch, use_half):
    count = 300_000 + 3
    g = synth.rng(int(epoch * 100) + use_half)
    theta = synth.normal(g, count, 0.05)
    delta = synth.normal(g, count, 1e-3)
    m = synth.normal(g, count, 1e-3) ** 2
    grad = synth.gradient_like(g, count)
    eta = 6.4
    a_sgd = rn.rn50_alpha_sgd(epoch)
    a_rms = rn.rn50_alpha_rmsprop(a_sgd, 3e-4, eta)
    assert abs(a_sgd - orc.alpha_sgd(epoch)) < 1e-15 and abs(a_rms - orc.alpha_rmsprop(a_sgd, 3e-4, eta)) < 1e-18
    mask_groups = (np.arange((count + 63) // 64) % 3 != 0).astype(np.uint8)
    decay = np.repeat(mask_groups, 64)[:count]
    hp = rn.opt_hparams(eta, 0.9, 0.99, 1e-8, a_sgd, a_rms, wd=1e-4, g_scale=1.0 / 1024 if use_half else 1.0)
    dth, dde, dm = to_dev(theta), to_dev(delta), to_dev(m)
    dmask = torch.from_numpy(mask_groups).to(DEV)
    if use_half:
        g16 = orc.grad_pack_fp16(grad * 1024)  # what the half-precision buffer would hold
        g_eff = orc.grad_unpack_fp16(g16, 1.0 / 1024)
        rn.opt_update(count, dth, dde, dm, None, torch.from_numpy(g16.view(np.int16)).to(DEV), dmask, hp)
    else:
        g_eff = grad.astype(np.float64)
        rn.opt_update(count, dth, dde, dm, to_dev(grad), None, dmask, hp)
    ok = np.isfinite(g_eff)
    rth, rde, rm = orc.opt_update(theta, delta, m, np.where(ok, g_eff, 0.0), eta, 0.9, 0.99, 1e-8, a_sgd, a_rms, 1e-4, decay)
    assert_close(dth.cpu().numpy()[ok], rth[ok], TOL, "theta")
    assert_close(dde.cpu().numpy()[ok], rde[ok], TOL, "delta")
    assert_close(dm.cpu().numpy()[ok], rm[ok], TOL, "m")


def test_opt_update_zero_state_and_no_mask():
    count = 4099
    g = synth.rng(5)
    theta, grad = synth.normal(g, count), synth.normal(g, count)
    hp = rn.opt_hparams(0.1, 0.9, 0.99, 1e-8, 1.0, 0.0, wd=1e-4)
    dth, dde, dm = to_dev(theta), to_dev(np.zeros(count)), to_dev(np.zeros(count))
    rn.opt_update(count, dth, dde, dm, to_dev(grad), None, None, hp)
    rth, rde, rm = orc.opt_update(theta, np.zeros(count), np.zeros(count), grad, 0.1, 0.9, 0.99, 1e-8, 1.0, 0.0, 1e-4, None)
    assert_close(dth.cpu().numpy(), rth, TOL, "theta")
    assert_close(dde.cpu().numpy(), rde, TOL, "delta")
    assert_close(dm.cpu().numpy(), rm, TOL, "m")
    # momentum-SGD closed form of the one-block configuration: theta1 = theta0 - 0.1*(g + 1e-4*theta0)
    assert_close(dth.cpu().numpy(), theta.astype(np.float64) - 0.1 * (grad + 1e-4 * theta.astype(np.float64)), TOL, "closed form")


def test_opt_update_argument_errors():
    hp = rn.opt_hparams(0.1)
    t = empty(64)
    with pytest.raises(rn.Rn50Error) as e:
        rn.opt_update(64, t, t, t, None, None, None, hp)
    assert e.value.code == rn.EINVAL
    with pytest.raises(rn.Rn50Error):
        rn.opt_update(64, t, t, t, t, t, None, hp)
