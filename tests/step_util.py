"""Shared pieces of the whole-step GPU tests: parameter marshalling between the oracle's {name: KCRS array}
dict and the library's flat KRSC arenas, and a runner for both sides."""
import numpy as np
import torch

from oracle import resnet50
from paper_1711_04325_amd import binding as rn
from paper_1711_04325_amd import synth
from tests.gpu_util import DEV


def flat_from_dict(tensors, dtype=np.float32):
    """{name: logical array} -> flat arena in the library's order and layout (filters KRSC)."""
    parts = []
    for name, off, cnt, dims, kind in rn.rn50_param_table():
        a = np.asarray(tensors[name])
        if kind == 0:
            a = np.transpose(a, (0, 2, 3, 1))
        parts.append(np.ascontiguousarray(a, dtype=dtype).ravel())
        assert parts[-1].size == cnt
    return np.concatenate(parts)


def dict_from_flat(flat):
    """flat arena (library order/layout) -> {name: logical array (filters KCRS)} of float64"""
    out = {}
    for name, off, cnt, dims, kind in rn.rn50_param_table():
        a = np.asarray(flat[off:off + cnt], dtype=np.float64)
        if kind == 0:
            k, r, s, c = dims
            a = np.transpose(a.reshape(k, r, s, c), (0, 3, 1, 2))
        elif kind == 3:
            a = a.reshape(dims[0], dims[1])
        out[name] = a
    return out


def problem(seed, batch, perturb_bn=True):
    g = synth.rng(seed)
    images = synth.normal(g, (batch, 3, 224, 224))
    params = synth.params(g, resnet50.param_table(), perturb_bn=perturb_bn)
    labels = synth.labels(g, batch)
    return images, params, labels


def gpu_forward_backward(ctx, images, params, labels, bn_eps):
    dimg = torch.from_numpy(np.ascontiguousarray(images.transpose(0, 2, 3, 1))).to(DEV)
    dlab = torch.from_numpy(labels).to(DEV)
    theta = torch.from_numpy(flat_from_dict(params)).to(DEV)
    grad = torch.empty_like(theta)
    loss = torch.empty(1, device=DEV)
    ctx.forward_backward(dimg, dlab, theta, grad, bn_eps, loss)
    torch.cuda.synchronize()
    return loss.item(), grad, theta, dimg, dlab
