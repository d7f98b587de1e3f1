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


def bottleneck_fwd_bwd(params, x, dout, name, stride=1, project=True, eps=2e-5, keep=None, masks=None):
    """One bottleneck block: a 1x1 -> BN+ReLU, b 3x3 -> BN+ReLU, c 1x1 -> BN, shortcut (projection 1x1 -> BN,
    or identity), sum, ReLU.  Returns (out, dx, grads).  masks: optional {layer name: array} whose signs
    replace the stored forward outputs as ReLU masks in the backward (diagnostic for sign flips)."""
    masks = masks or {}
    a = _ConvBN(name + ".a", stride, 0, True)
    b = _ConvBN(name + ".b", 1, 1, True)
    c = _ConvBN(name + ".c", 1, 0, True)
    p = _ConvBN(name + ".p", stride, 0, False) if project else None
    shortcut = p.fwd(params, x, eps, keep=keep) if project else x
    out = c.fwd(params, b.fwd(params, a.fwd(params, x, eps, keep=keep), eps, keep=keep), eps, residual=shortcut,
                keep=keep)
    grads = {}
    d, dshort = c.bwd(grads, dout, relu_mask_from=masks.get(name + ".c"))
    d, _ = b.bwd(grads, d, relu_mask_from=masks.get(name + ".b"))
    dx, _ = a.bwd(grads, d, relu_mask_from=masks.get(name + ".a"))
    if project:
        dxp, _ = p.bwd(grads, dshort)
        dx = dx + dxp
    else:
        dx = dx + dshort
    return out, dx, grads


def wiring(variant="v1"):
    """Data flow of the network, one entry per convolution in forward order:
    (name, input tensor name, residual tensor name or None, relu, stride, pad).  Tensor names: "images",
    "pool.out", "<layer>.out"."""
    layers = {l[0]: l for l in conv_layers(variant)}
    w = [("stem", "images", None, True, 2, 3)]
    block_in = "pool.out"
    for si, (width, nblocks, _) in enumerate(STAGES):
        for bi in range(nblocks):
            name = "s%d.b%d" % (si + 2, bi)
            shortcut = block_in
            if bi == 0:
                w.append((name + ".p", block_in, None, False, layers[name + ".p"][4], 0))
                shortcut = name + ".p.out"
            w.append((name + ".a", block_in, None, True, layers[name + ".a"][4], 0))
            w.append((name + ".b", name + ".a.out", None, True, layers[name + ".b"][4], 1))
            w.append((name + ".c", name + ".b.out", shortcut, True, 1, 0))
            block_in = name + ".c.out"
    return w


class State:
    """Everything the backward pass needs: per-layer _ConvBN records, pooling indices, head tensors."""


def forward(params, images, labels, eps=2e-5, variant="v1", keep=None):
    st = State()
    st.variant = variant
    t = {"images": np.asarray(images, dtype=np.float64)}
    st.layers = {}
    for name, src, res, relu, stride, pad in wiring(variant):
        l = _ConvBN(name, stride, pad, relu)
        t[name + ".out"] = l.fwd(params, t[src], eps, residual=t[res] if res else None, keep=keep)
        st.layers[name] = l
        if name == "stem":
            st.pool_in_shape = t["stem.out"].shape
            t["pool.out"], st.pool_arg = ops.maxpool_fwd(t["stem.out"], 3, 2, 1)
            if keep is not None:
                keep["pool.out"], keep["pool.arg"] = t["pool.out"], st.pool_arg
        last = name
    h = t[last + ".out"]
    st.feat_shape = h.shape
    st.feat = ops.avgpool_fwd(h)
    st.logits = ops.fc_fwd(st.feat, params["fc.w"], params["fc.b"])
    st.loss, st.dlogits = ops.softmax_ce(st.logits, labels)
    if keep is not None:
        keep["feat"], keep["logits"], keep["dlogits"] = st.feat, st.logits, st.dlogits
    return st


def forward_eval(params, images, stats, variant="v1"):
    """Validation-side forward: every BN normalises with the given statistics (stats[name + ".mean"],
    stats[name + ".invstd"]: the last training minibatch's, averaged over the workers; Section 2).  Returns logits."""
    t = {"images": np.asarray(images, dtype=np.float64)}
    for name, src, res, relu, stride, pad in wiring(variant):
        conv = ops.conv2d_fwd(t[src], params[name + ".w"], stride, pad)
        t[name + ".out"] = ops.bn_inference(conv, params[name + ".g"], params[name + ".beta"], stats[name + ".mean"],
                                            stats[name + ".invstd"], residual=t[res] if res else None, relu=relu)
        if name == "stem":
            t["pool.out"], _ = ops.maxpool_fwd(t["stem.out"], 3, 2, 1)
        last = name
    return ops.fc_fwd(ops.avgpool_fwd(t[last + ".out"]), params["fc.w"], params["fc.b"])


def backward(st, params):
    """Gradients of the loss with respect to every parameter, from a forward State."""
    grads = {}
    df, grads["fc.w"], grads["fc.b"] = ops.fc_bwd(st.feat, params["fc.w"], st.dlogits)
    acc = {}  # gradient accumulated on each activation tensor, by name

    def add(name, g):
        acc[name] = g if name not in acc else acc[name] + g

    w = wiring(st.variant)
    add(w[-1][0] + ".out", ops.avgpool_bwd(df, st.feat_shape[2], st.feat_shape[3]))
    for name, src, res, relu, stride, pad in reversed(w):
        if name == "stem":
            d = ops.maxpool_bwd(acc.pop("pool.out"), st.pool_arg, st.pool_in_shape[2], st.pool_in_shape[3], 3, 2, 1)
            st.layers[name].bwd(grads, d, need_dx=False)
            break
        dx, dres = st.layers[name].bwd(grads, acc.pop(name + ".out"))
        add(src, dx)
        if res:
            add(res, dres)
    return grads


def forward_backward(params, images, labels, eps=2e-5, variant="v1", keep=None):
    """Forward, loss and backward of the whole network.  Returns (loss, grads dict of float64)."""
    st = forward(params, images, labels, eps, variant, keep)
    return st.loss, backward(st, params)


def state_from_saved(params, images, labels, saved, variant="v1"):
    """A State whose forward tensors are GIVEN (e.g. the fp32 tensors a device run stored) instead of computed:
    saved[name + ".conv" | ".out" | ".mean" | ".invstd"], saved["pool.out"], saved["pool.arg"] (flat h*W+w
    indices), saved["feat"], saved["logits"].  backward() on it is then a linear map of the head gradient with
    the same ReLU masks, arg-max choices and normalisation statistics as the run that produced the tensors."""
    st = State()
    st.variant = variant
    t = {"images": np.asarray(images, dtype=np.float64), "pool.out": np.asarray(saved["pool.out"], dtype=np.float64)}
    for name, *_ in wiring(variant):
        t[name + ".out"] = np.asarray(saved[name + ".out"], dtype=np.float64)
    st.layers = {}
    for name, src, res, relu, stride, pad in wiring(variant):
        l = _ConvBN(name, stride, pad, relu)
        l.x, l.w, l.gamma = t[src], params[name + ".w"], params[name + ".g"]
        l.conv_out = np.asarray(saved[name + ".conv"], dtype=np.float64)
        l.y, l.has_res = t[name + ".out"], res is not None
        l.mean = np.asarray(saved[name + ".mean"], dtype=np.float64)
        l.invstd = np.asarray(saved[name + ".invstd"], dtype=np.float64)
        st.layers[name] = l
        last = name
    st.pool_in_shape = t["stem.out"].shape
    st.pool_arg = np.asarray(saved["pool.arg"], dtype=np.int32)
    st.feat_shape = t[last + ".out"].shape
    st.feat = np.asarray(saved["feat"], dtype=np.float64)
    st.logits = np.asarray(saved["logits"], dtype=np.float64)
    st.loss, st.dlogits = ops.softmax_ce(st.logits, labels)
    return st


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
