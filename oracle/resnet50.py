"""ResNet-50 training step composed from the oracle's fp64 primitives.

Test infrastructure only.  The architecture is He et al. 2016's ResNet-50 ("v1": the
stride of 2 sits on the first 1x1 convolution of the first block of stages 3-5), which
the paper trains (Section 1) with a per-worker minibatch of 32 (Section 4); batch
normalization uses the current minibatch's statistics only (Section 2); the update is
the rule of Appendix A.1 applied to gradients that went through the half-precision
communication buffer (Section 3, "Software").

Tensors are logical NCHW / KCRS float64 numpy arrays.  Parameters live in a dict keyed
by the names of `param_table()`; the flat order of that table is the order of the
half-precision communication buffer.
"""
import numpy as np

from . import ops

STAGES = ((64, 3, 1), (128, 4, 2), (256, 6, 2), (512, 3, 2))  # (width, blocks, stride of first block)
NUM_CLASSES = 1000


def conv_layers(variant="v1"):
    """[(name, C, K, R, stride, pad, H_in)] for the 53 convolutions in forward order."""
    out = [("stem", 3, 64, 7, 2, 3, 224)]
    cin, h = 64, 56
    for si, (width, nblocks, stride0) in enumerate(STAGES):
        for bi in range(nblocks):
            stride = stride0 if bi == 0 else 1
            sa, sb = (stride, 1) if variant == "v1" else (1, stride)
            name = "s%d.b%d" % (si + 2, bi)
            out.append((name + ".a", cin, width, 1, sa, 0, h))
            out.append((name + ".b", width, width, 3, sb, 1, h // sa))
            out.append((name + ".c", width, 4 * width, 1, 1, 0, h // stride))
            if bi == 0:
                out.append((name + ".p", cin, 4 * width, 1, stride, 0, h))
            cin, h = 4 * width, h // stride
    return out


def param_table(variant="v1"):
    """[(name, shape, kind)] in communication-buffer order; kind in conv_w, bn_g, bn_b, fc_w, fc_b."""
    t = []
    for name, c, k, r, _, _, _ in conv_layers(variant):
        t.append((name + ".w", (k, c, r, r), "conv_w"))
        t.append((name + ".g", (k,), "bn_g"))
        t.append((name + ".beta", (k,), "bn_b"))
    t.append(("fc.w", (NUM_CLASSES, 2048), "fc_w"))
    t.append(("fc.b", (NUM_CLASSES,), "fc_b"))
    return t


def param_count(variant="v1"):
    return sum(int(np.prod(s)) for _, s, _ in param_table(variant))


def conv_macs_per_image(variant="v1"):
    tot = 0
    for _, c, k, r, stride, pad, h in conv_layers(variant):
        p = ops.out_size(h, r, stride, pad)
        tot += c * k * r * r * p * p
    return tot


class _ConvBN:
    """conv -> BN(batch statistics) [+ residual] [-> ReLU], with everything the backward needs."""

    def __init__(self, name, stride, pad, relu):
        self.name, self.stride, self.pad, self.relu = name, stride, pad, relu

    def fwd(self, params, x, eps, residual=None, keep=None):
        self.x = x
        self.w = params[self.name + ".w"]
        self.gamma = params[self.name + ".g"]
        self.conv_out = ops.conv2d_fwd(x, self.w, self.stride, self.pad)
        self.has_res = residual is not None
        self.y, self.mean, self.invstd = ops.bn_fwd(self.conv_out, self.gamma, params[self.name + ".beta"], eps,
                                                    residual=residual, relu=self.relu)
        if keep is not None:
            keep[self.name + ".conv"] = self.conv_out
            keep[self.name + ".out"] = self.y
            keep[self.name + ".mean"] = self.mean
            keep[self.name + ".invstd"] = self.invstd
        return self.y

    def bwd(self, grads, dy, need_dx=True, relu_mask_from=None):
        """Returns (dx or None, dresidual or None).  relu_mask_from replaces the stored forward output
        as the source of the ReLU mask (a diagnostic: attribute parity excess to sign flips)."""
        y = self.y if relu_mask_from is None else relu_mask_from
        dconv, dres, dg, db = ops.bn_bwd(self.conv_out, dy, y if self.relu else None, self.gamma, self.mean,
                                         self.invstd, relu=self.relu, want_dresidual=self.has_res)
        grads[self.name + ".g"] = dg
        grads[self.name + ".beta"] = db
        r = self.w.shape[2]
        grads[self.name + ".w"] = ops.conv2d_bwd_weight(self.x, dconv, r, r, self.stride, self.pad)
        dx = None
        if need_dx:
            dx = ops.conv2d_bwd_data(dconv, self.w, self.stride, self.pad, self.x.shape[2], self.x.shape[3])
        return dx, dres


def bottleneck_fwd_bwd(params, x, dout, name, stride=1, project=True, eps=2e-5, keep=None):
    """One bottleneck block: a 1x1 -> BN+ReLU, b 3x3 -> BN+ReLU, c 1x1 -> BN, shortcut (projection 1x1 -> BN,
    or identity), sum, ReLU.  Returns (out, dx, grads)."""
    a = _ConvBN(name + ".a", stride, 0, True)
    b = _ConvBN(name + ".b", 1, 1, True)
    c = _ConvBN(name + ".c", 1, 0, True)
    p = _ConvBN(name + ".p", stride, 0, False) if project else None
    shortcut = p.fwd(params, x, eps, keep=keep) if project else x
    out = c.fwd(params, b.fwd(params, a.fwd(params, x, eps, keep=keep), eps, keep=keep), eps, residual=shortcut,
                keep=keep)
    grads = {}
    d, dshort = c.bwd(grads, dout)
    d, _ = b.bwd(grads, d)
    dx, _ = a.bwd(grads, d)
    if project:
        dxp, _ = p.bwd(grads, dshort)
        dx = dx + dxp
    else:
        dx = dx + dshort
    return out, dx, grads


def forward_backward(params, images, labels, eps=2e-5, variant="v1", keep=None):
    """Forward, loss and backward of the whole network.  Returns (loss, grads dict of float64)."""
    layers = {l[0]: l for l in conv_layers(variant)}
    stem = _ConvBN("stem", 2, 3, True)
    h = stem.fwd(params, images, eps, keep=keep)
    pool_in_shape = h.shape
    h, arg = ops.maxpool_fwd(h, 3, 2, 1)
    if keep is not None:
        keep["pool.out"] = h
    blocks = []
    for si, (width, nblocks, _) in enumerate(STAGES):
        for bi in range(nblocks):
            name = "s%d.b%d" % (si + 2, bi)
            a = _ConvBN(name + ".a", layers[name + ".a"][4], 0, True)
            b = _ConvBN(name + ".b", layers[name + ".b"][4], 1, True)
            c = _ConvBN(name + ".c", 1, 0, True)
            p = _ConvBN(name + ".p", layers[name + ".p"][4], 0, False) if bi == 0 else None
            shortcut = p.fwd(params, h, eps, keep=keep) if p else h
            h = c.fwd(params, b.fwd(params, a.fwd(params, h, eps, keep=keep), eps, keep=keep), eps,
                      residual=shortcut, keep=keep)
            blocks.append((a, b, c, p))
    feat_shape = h.shape
    f = ops.avgpool_fwd(h)
    logits = ops.fc_fwd(f, params["fc.w"], params["fc.b"])
    loss, dlogits = ops.softmax_ce(logits, labels)
    if keep is not None:
        keep["feat"] = f
        keep["logits"] = logits

    grads = {}
    df, grads["fc.w"], grads["fc.b"] = ops.fc_bwd(f, params["fc.w"], dlogits)
    d = ops.avgpool_bwd(df, feat_shape[2], feat_shape[3])
    for a, b, c, p in reversed(blocks):
        dc, dshort = c.bwd(grads, d)
        db_, _ = b.bwd(grads, dc)
        dx, _ = a.bwd(grads, db_)
        if p:
            dxp, _ = p.bwd(grads, dshort)
            d = dx + dxp
        else:
            d = dx + dshort
    d = ops.maxpool_bwd(d, arg, pool_in_shape[2], pool_in_shape[3], 3, 2, 1)
    stem.bwd(grads, d, need_dx=False)
    return loss, grads


def flatten(tensors, variant="v1", dtype=np.float64):
    return np.concatenate([np.asarray(tensors[n], dtype=dtype).ravel() for n, _, _ in param_table(variant)])


def unflatten(flat, variant="v1"):
    out, o = {}, 0
    for n, s, _ in param_table(variant):
        c = int(np.prod(s))
        out[n] = flat[o:o + c].reshape(s)
        o += c
    return out


def decay_mask(variant="v1"):
    """1 where L2 weight decay applies: convolution and FC weights, not BN scale/shift, not the FC bias."""
    return np.concatenate([np.full(int(np.prod(s)), 1 if kind in ("conv_w", "fc_w") else 0, dtype=np.uint8)
                           for _, s, kind in param_table(variant)])


def communicate_and_update(theta, delta, m, grads32, hp, n_workers=1024, variant="v1"):
    """Pack the fp32 gradient to half precision, (the all-reduce of a single worker is the identity,)
    unpack with scale 1/n_workers, apply the update rule.  All flat arrays in table order.
    hp: dict(eta, mu1, mu2, eps, a_sgd, a_rms, wd).  Returns (g16, g_unpacked, theta, delta, m)."""
    g16 = ops.grad_pack_fp16(np.asarray(grads32, dtype=np.float32))
    g = ops.grad_unpack_fp16(g16, 1.0 / n_workers)
    th, de, mm = ops.opt_update(theta, delta, m, g, hp["eta"], hp["mu1"], hp["mu2"], hp["eps"], hp["a_sgd"],
                                hp["a_rms"], hp.get("wd", 0.0), decay_mask(variant))
    return g16, g, th, de, mm
