"""Shared pieces of the whole-step GPU tests: parameter marshalling between the oracle's {name: KCRS array}
dict and the library's flat KRSC arenas, and a runner for both sides."""
import numpy as np
import torch

from oracle import resnet50
from paper_1711_04325_amd import binding as rn
from paper_1711_04325_amd.arena import dict_from_flat, flat_from_dict  # noqa: F401 (re-exported)
from paper_1711_04325_amd import synth
from tests.gpu_util import DEV


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
