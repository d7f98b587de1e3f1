"""Helpers of the GPU parity tests: layout conversion between the oracle's logical NCHW / KCRS arrays and the
library's NHWC / KRSC device tensors, and the parity metric."""
import numpy as np
import torch

DEV = "cuda:0"
TOL = 1e-4  # rel-L2 bar for fp32 outputs and gradients against the fp64 oracle


def to_dev(a, dtype=torch.float32):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV).to(dtype).contiguous()


def nhwc(a):
    """logical NCHW (or KCRS) numpy -> device NHWC (KRSC) fp32 tensor"""
    return to_dev(np.ascontiguousarray(np.transpose(a, (0, 2, 3, 1)), dtype=np.float32))


def nchw(t):
    """device NHWC (KRSC) tensor -> logical NCHW (KCRS) float64 numpy"""
    return np.transpose(t.detach().cpu().numpy().astype(np.float64), (0, 3, 1, 2))


def empty(*shape, dtype=torch.float32):
    return torch.empty(shape, dtype=dtype, device=DEV)


def ws_bytes(nbytes):
    """A kernel workspace (scratch; zero-filled only so that a kernel that reads before writing would show)."""
    return torch.zeros(max(int(nbytes), 16), dtype=torch.uint8, device=DEV)


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    nr = np.linalg.norm(ref)
    d = np.linalg.norm(got - ref)
    if nr == 0.0:
        return d / (1e-6 * np.sqrt(max(ref.size, 1))) * TOL  # absolute bar 1e-6*sqrt(count) mapped onto TOL
    return d / nr


def assert_close(got, ref, tol=TOL, what=""):
    e = rel_l2(got, ref)
    assert np.all(np.isfinite(np.asarray(got, dtype=np.float64))), what + ": non-finite values"
    assert e <= tol, "%s: rel-L2 %.3e > %.1e" % (what, e, tol)
    return e


def bf16_round(a):
    """Nearest bf16 value (8 significant bits, ties to even) of every element, as float64; written with frexp /
    rint so that it shares nothing with the integer bit trick a kernel would use.  Normal range only."""
    m, e = np.frexp(np.asarray(a, dtype=np.float32).astype(np.float64))
    return np.ldexp(np.rint(np.ldexp(m, 8)), e - 8)
