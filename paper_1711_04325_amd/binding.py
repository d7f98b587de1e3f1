"""Thin ctypes binding of librn50.so: same names as the C ABI in include/rn50.h, argument marshalling only.

Tensor arguments are torch tensors on the GPU (contiguous; NHWC activations, KRSC filters); they are
passed as raw device pointers.  torch supplies device memory and the current stream, nothing else:
every arithmetic step runs in the library's kernels.  There is no fallback: if the library is missing
or a call fails, an exception is raised.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("RN50_LIB") or os.path.join(_HERE, "librn50.so")  # RN50_LIB: an alternative build (measurements)

OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP = 0, -1, -2, -3, -4
LAYOUT_NCHW, LAYOUT_NHWC = 0, 1
DTYPE_F32, DTYPE_BF16, DTYPE_BF16_ACT, DTYPE_BF16_ACT_F32IN = 0, 1, 2, 3
VARIANT_V1, VARIANT_V15 = 0, 1
OP_FWD, OP_BWD_DATA, OP_BWD_WEIGHT, OP_BWD_DATA_FLIPPED, OP_FWD_BNSTATS = 0, 1, 2, 3, 4
WD_GROUP = 64
KIND_NAMES = {0: "conv_w", 1: "bn_g", 2: "bn_b", 3: "fc_w", 4: "fc_b"}


class Rn50Error(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("librn50 error %d: %s" % (code, msg))
        self.code = code


class ConvDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("n", "c", "h", "w", "k", "r", "s", "stride", "pad", "layout", "in_dtype")]


class WgradGroupItem(C.Structure):
    _fields_ = [("desc", ConvDesc), ("x", C.c_void_p), ("in_scale", C.c_void_p), ("in_shift", C.c_void_p), ("dy", C.c_void_p),
                ("dw_offset", C.c_size_t)]


class OptHparams(C.Structure):
    _fields_ = [(n, C.c_float) for n in ("eta", "mu1", "mu2", "eps", "a_sgd", "a_rms", "wd", "g_scale")]


_vp, _sz, _i, _f = C.c_void_p, C.c_size_t, C.c_int, C.c_float
_SIGS = {
    "rn50_last_error": (C.c_char_p, []),
    "rn50_set_option": (_i, [C.c_char_p, C.c_char_p]),
    "rn50_conv_workspace_bytes": (_sz, [C.POINTER(ConvDesc), _i]),
    "rn50_conv_plan": (_i, [C.POINTER(ConvDesc), _i, C.POINTER(_i), C.POINTER(_i), C.POINTER(_i), C.POINTER(_i)]),
    "rn50_probe_mfma": (_i, [_i, _i, _i, _vp, _vp, C.POINTER(C.c_double), _vp]),
    "rn50_probe_copy": (_i, [_sz, _vp, _vp, _vp]),
    "rn50_probe_empty": (_i, [_i, _i, _vp, _vp]),
    "conv2d_fwd": (_i, [C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _sz, _vp]),
    "conv2d_bwd_data": (_i, [C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _sz, _vp]),
    "conv2d_bwd_weight": (_i, [C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _sz, _vp]),
    "conv2d_filter_flip": (_i, [C.POINTER(ConvDesc), _vp, _vp, _vp]),
    "conv2d_bwd_data_flipped": (_i, [C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _sz, _vp]),
    "conv2d_fwd_bnrelu_input": (_i, [C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "conv2d_bwd_weight_bnrelu_input": (_i, [C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "rn50_wgrad_group_table_bytes": (_sz, [_i]),
    "rn50_wgrad_group_workspace_bytes": (_sz, [_i, C.POINTER(WgradGroupItem)]),
    "rn50_wgrad_group_plan": (_i, [_i, C.POINTER(WgradGroupItem), _vp, _sz, _vp, _sz]),
    "conv2d_bwd_weight_group": (_i, [_vp, _vp, _vp, _vp]),
    "conv2d_fwd_bnstats": (_i, [C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _f, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "bn_fwd_apply": (_i, [_i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _i, _vp, _vp, _vp]),
    "bn_fwd_apply_bf16": (_i, [_i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _i, _vp, _vp, _vp]),
    "rn50_bn_workspace_bytes": (_sz, [_i, _i, _i, _i]),
    "bn_fwd_batchstats": (_i, [_i, _i, _i, _i, _i, _vp, _vp, _vp, _f, _vp, _i, _vp, _vp, _vp, _vp, _sz, _vp]),
    "bn_fwd_batchstats_static": (_i, [_i, _i, _i, _i, _i, _vp, _vp, _vp, _f, _vp, _i, _vp, _vp, _vp, _vp]),
    "bn_bwd_batchstats": (_i, [_i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "bn_fwd_batchstats_mask": (_i, [_i, _i, _i, _i, _i, _vp, _vp, _vp, _f, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "bn_bwd_batchstats_mask": (_i, [_i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "bn_stats_scale_shift": (_i, [_i, _i, _i, _i, _i, _vp, _vp, _vp, _f, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "bn_bwd_batchstats_xmask": (_i, [_i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "bn_fwd_batchstats_bf16": (_i, [_i, _i, _i, _i, _i, _vp, _vp, _vp, _f, _vp, _i, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "bn_stats_scale_shift_bf16": (_i, [_i, _i, _i, _i, _i, _vp, _vp, _vp, _f, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "bn_bwd_batchstats_bf16": (_i, [_i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "maxpool3x3s2_fwd_bf16": (_i, [_i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp]),
    "maxpool3x3s2_bwd_bf16": (_i, [_i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp]),
    "avgpool_fwd_bf16": (_i, [_i, _i, _i, _i, _vp, _vp, _vp]),
    "avgpool_bwd_bf16": (_i, [_i, _i, _i, _i, _vp, _vp, _vp]),
    "bn_fwd_inference": (_i, [_i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _i, _vp, _vp, _sz, _vp]),
    "bn_stats_average": (_i, [_i, _i, _vp, _vp, _f, _vp, _vp, _vp]),
    "maxpool3x3s2_fwd": (_i, [_i, _i, _i, _i, _vp, _vp, _vp, _vp]),
    "maxpool3x3s2_bwd": (_i, [_i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp]),
    "maxpool3x3s2_fwd_bnrelu_input": (_i, [_i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp]),
    "avgpool_fwd": (_i, [_i, _i, _i, _i, _vp, _vp, _vp]),
    "avgpool_bwd": (_i, [_i, _i, _i, _i, _vp, _vp, _vp]),
    "fc_fwd": (_i, [_i, _i, _i, _vp, _vp, _vp, _vp, _vp]),
    "fc_bwd": (_i, [_i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "softmax_ce": (_i, [_i, _i, _vp, _vp, _vp, _vp, _vp]),
    "grad_pack_fp16": (_i, [_sz, _vp, _vp, _vp]),
    "grad_unpack_fp16": (_i, [_sz, _vp, _f, _vp, _vp]),
    "opt_update": (_i, [_sz, _vp, _vp, _vp, _vp, _vp, _vp, C.POINTER(OptHparams), _vp]),
    "rn50_alpha_sgd": (C.c_double, [C.c_double, C.c_double, C.c_double]),
    "rn50_alpha_sgd_transition": (C.c_double, [C.c_double, C.c_double, C.c_double, _i]),
    "rn50_alpha_rmsprop": (C.c_double, [C.c_double, C.c_double, C.c_double]),
    "rn50_lr_base": (C.c_double, [_i, _i]),
    "rn50_lr_slow_start": (C.c_double, [C.c_double, _i, _i]),
    "rn50_recipe_hparams": (_i, [C.c_double, _i, _i, C.POINTER(OptHparams)]),
    "rn50_recipe_hparams_transition": (_i, [C.c_double, _i, _i, _i, C.POINTER(OptHparams)]),
    "rn50_param_count": (_sz, []),
    "rn50_param_table_size": (_i, []),
    "rn50_param_table": (_i, [_i, C.POINTER(C.c_char_p), C.POINTER(_sz), C.POINTER(_sz), C.POINTER(_i * 4), C.POINTER(_i)]),
    "rn50_activation_bytes": (_sz, [_i, _i]),
    "rn50_create": (_i, [C.POINTER(_vp), _i, _i, _i, _vp, _sz]),
    "rn50_destroy": (None, [_vp]),
    "rn50_step": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, C.POINTER(OptHparams), _f, _vp, _vp]),
    "rn50_forward_backward": (_i, [_vp, _vp, _vp, _vp, _vp, _f, _vp, _vp]),
    "rn50_peek": (_vp, [_vp, _i, _i, C.POINTER(_sz), _vp]),
    "rn50_filter_flip_all": (_i, [_vp, _vp, _vp]),
    "rn50_wgrad_groups_run": (_i, [_vp, _vp, _vp]),
    "rn50_forward_eval": (_i, [_vp, _vp, _vp, _vp, _vp]),
    "rn50_set_bn_stats": (_i, [_vp, _i, _vp, _vp, _vp]),
}
EXPORTS = tuple(_SIGS)

_lib = None


def lib():
    """Loads librn50.so (built in-tree by paper_1711_04325_amd.build); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError("%s is missing: run `python -m paper_1711_04325_amd.build`" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise Rn50Error(rc, lib().rn50_last_error().decode())


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous GPU tensors"
    return t.data_ptr()


def _stream(stream=None):
    return stream if stream is not None else torch.cuda.current_stream().cuda_stream


def conv_desc(n, c, h, w, k, r, s, stride, pad, layout=LAYOUT_NHWC, in_dtype=DTYPE_F32):
    return ConvDesc(n, c, h, w, k, r, s, stride, pad, layout, in_dtype)


def rn50_last_error():
    return lib().rn50_last_error().decode()


def rn50_set_option(name, value=None):
    """Tuning / test switch (see include/rn50.h); value None restores the built-in default."""
    _check(lib().rn50_set_option(name.encode(), None if value is None else str(value).encode()))


def rn50_conv_workspace_bytes(desc, op):
    return lib().rn50_conv_workspace_bytes(C.byref(desc), op)


def rn50_conv_plan(desc, op):
    """(bm, bn, split, workgroups) of the launch the library would use."""
    v = [_i() for _ in range(4)]
    _check(lib().rn50_conv_plan(C.byref(desc), op, *[C.byref(t) for t in v]))
    return tuple(t.value for t in v)


def rn50_probe_mfma(dtype, iters, wgs_per_cu, sink, ticks=None, stream=None):
    """Enqueues the pure-MFMA loop; returns the floating-point operations of the launch.  ticks: two device int64
    (shader-clock cycles, 100 MHz reference ticks of the first wavefront's loop) or None."""
    flop = C.c_double()
    _check(lib().rn50_probe_mfma(dtype, iters, wgs_per_cu, _ptr(sink), _ptr(ticks), C.byref(flop), _stream(stream)))
    return flop.value


def rn50_probe_copy(count, src, dst, stream=None):
    _check(lib().rn50_probe_copy(count, _ptr(src), _ptr(dst), _stream(stream)))


def rn50_probe_empty(workgroups, launches=1, sink=None, stream=None):
    _check(lib().rn50_probe_empty(workgroups, launches, _ptr(sink), _stream(stream)))


def _bytes(ws):
    return 0 if ws is None else ws.numel() * ws.element_size()


def conv2d_fwd(desc, x, w, y, ws=None, stream=None):
    _check(lib().conv2d_fwd(C.byref(desc), _ptr(x), _ptr(w), _ptr(y), _ptr(ws), _bytes(ws), _stream(stream)))


def conv2d_bwd_data(desc, dy, w, dx, ws=None, stream=None):
    _check(lib().conv2d_bwd_data(C.byref(desc), _ptr(dy), _ptr(w), _ptr(dx), _ptr(ws), _bytes(ws), _stream(stream)))


def conv2d_filter_flip(desc, w, wt, stream=None):
    _check(lib().conv2d_filter_flip(C.byref(desc), _ptr(w), _ptr(wt), _stream(stream)))


def conv2d_bwd_data_flipped(desc, dy, wt, dx, ws=None, stream=None):
    _check(lib().conv2d_bwd_data_flipped(C.byref(desc), _ptr(dy), _ptr(wt), _ptr(dx), _ptr(ws), _bytes(ws), _stream(stream)))


def conv2d_bwd_weight(desc, x, dy, dw, ws=None, stream=None):
    _check(lib().conv2d_bwd_weight(C.byref(desc), _ptr(x), _ptr(dy), _ptr(dw), _ptr(ws), _bytes(ws), _stream(stream)))


def conv2d_fwd_bnrelu_input(desc, x, in_scale, in_shift, w, y, ws=None, stream=None):
    _check(lib().conv2d_fwd_bnrelu_input(C.byref(desc), _ptr(x), _ptr(in_scale), _ptr(in_shift), _ptr(w), _ptr(y), _ptr(ws), _bytes(ws),
                                         _stream(stream)))


def conv2d_bwd_weight_bnrelu_input(desc, x, in_scale, in_shift, dy, dw, ws=None, stream=None):
    _check(lib().conv2d_bwd_weight_bnrelu_input(C.byref(desc), _ptr(x), _ptr(in_scale), _ptr(in_shift), _ptr(dy), _ptr(dw), _ptr(ws),
                                                _bytes(ws), _stream(stream)))


def wgrad_group_items(layers):
    """layers: (desc, x, in_scale or None, in_shift or None, dy, dw_offset) per layer -> ctypes array of rn50_wgrad_group_item."""
    arr = (WgradGroupItem * len(layers))()
    for it, (desc, x, sc, sh, dy, off) in zip(arr, layers):
        it.desc, it.x, it.in_scale, it.in_shift, it.dy, it.dw_offset = desc, _ptr(x), _ptr(sc), _ptr(sh), _ptr(dy), off
    return arr


def rn50_wgrad_group_table_bytes(count):
    return lib().rn50_wgrad_group_table_bytes(count)


def rn50_wgrad_group_workspace_bytes(items):
    return lib().rn50_wgrad_group_workspace_bytes(len(items), items)


def rn50_wgrad_group_plan(items, ws):
    """Writes the plan into a host buffer and returns it (a ctypes char array: the caller uploads the same bytes)."""
    table = C.create_string_buffer(rn50_wgrad_group_table_bytes(len(items)))
    _check(lib().rn50_wgrad_group_plan(len(items), items, _ptr(ws), _bytes(ws), table, len(table)))
    return table


def conv2d_bwd_weight_group(table_host, table_device, dw_base, stream=None):
    _check(lib().conv2d_bwd_weight_group(table_host, _ptr(table_device), _ptr(dw_base), _stream(stream)))


def conv2d_fwd_bnstats(desc, x, in_scale, in_shift, w, y, gamma, beta, eps, save_mean, save_invstd, scale, shift, ws, stream=None):
    _check(lib().conv2d_fwd_bnstats(C.byref(desc), _ptr(x), _ptr(in_scale), _ptr(in_shift), _ptr(w), _ptr(y), _ptr(gamma), _ptr(beta), eps,
                                    _ptr(save_mean), _ptr(save_invstd), _ptr(scale), _ptr(shift), _ptr(ws), _bytes(ws), _stream(stream)))


def bn_fwd_apply(n, c, h, w, x, scale, shift, residual, relu, y, relu_mask=None, stream=None, layout=LAYOUT_NHWC):
    _check(lib().bn_fwd_apply(n, c, h, w, layout, _ptr(x), _ptr(scale), _ptr(shift), _ptr(residual), int(relu), _ptr(y), _ptr(relu_mask),
                              _stream(stream)))


def bn_fwd_apply_bf16(n, c, h, w, x, scale, shift, residual, relu, y, relu_mask=None, stream=None, layout=LAYOUT_NHWC):
    _check(lib().bn_fwd_apply_bf16(n, c, h, w, layout, _ptr(x), _ptr(scale), _ptr(shift), _ptr(residual), int(relu), _ptr(y),
                                   _ptr(relu_mask), _stream(stream)))


def rn50_bn_workspace_bytes(n, c, h, w):
    return lib().rn50_bn_workspace_bytes(n, c, h, w)


def bn_fwd_batchstats(n, c, h, w, x, gamma, beta, eps, residual, relu, y, save_mean, save_invstd, ws, stream=None,
                      layout=LAYOUT_NHWC):
    _check(lib().bn_fwd_batchstats(n, c, h, w, layout, _ptr(x), _ptr(gamma), _ptr(beta), eps, _ptr(residual), int(relu),
                                   _ptr(y), _ptr(save_mean), _ptr(save_invstd), _ptr(ws), _bytes(ws), _stream(stream)))


BN_STATIC_SCRATCH_BYTES = (2 * 512 + 4) * 2048 * 4


def bn_fwd_batchstats_static(n, c, h, w, x, gamma, beta, eps, residual, relu, y, save_mean, save_invstd, stream=None,
                             layout=LAYOUT_NHWC):
    _check(lib().bn_fwd_batchstats_static(n, c, h, w, layout, _ptr(x), _ptr(gamma), _ptr(beta), eps, _ptr(residual), int(relu),
                                          _ptr(y), _ptr(save_mean), _ptr(save_invstd), _stream(stream)))


def bn_fwd_batchstats_mask(n, c, h, w, x, gamma, beta, eps, residual, y, relu_mask, save_mean, save_invstd, ws, stream=None,
                           layout=LAYOUT_NHWC):
    _check(lib().bn_fwd_batchstats_mask(n, c, h, w, layout, _ptr(x), _ptr(gamma), _ptr(beta), eps, _ptr(residual), _ptr(y),
                                        _ptr(relu_mask), _ptr(save_mean), _ptr(save_invstd), _ptr(ws), _bytes(ws), _stream(stream)))


def bn_bwd_batchstats_mask(n, c, h, w, x, dy, dy2, relu_mask, gamma, save_mean, save_invstd, dx, dresidual, dgamma, dbeta, ws,
                           stream=None, layout=LAYOUT_NHWC):
    _check(lib().bn_bwd_batchstats_mask(n, c, h, w, layout, _ptr(x), _ptr(dy), _ptr(dy2), _ptr(relu_mask), _ptr(gamma), _ptr(save_mean),
                                        _ptr(save_invstd), _ptr(dx), _ptr(dresidual), _ptr(dgamma), _ptr(dbeta), _ptr(ws), _bytes(ws),
                                        _stream(stream)))


def bn_stats_scale_shift(n, c, h, w, x, gamma, beta, eps, save_mean, save_invstd, scale, shift, ws, stream=None, layout=LAYOUT_NHWC):
    _check(lib().bn_stats_scale_shift(n, c, h, w, layout, _ptr(x), _ptr(gamma), _ptr(beta), eps, _ptr(save_mean), _ptr(save_invstd),
                                      _ptr(scale), _ptr(shift), _ptr(ws), _bytes(ws), _stream(stream)))


def bn_bwd_batchstats_xmask(n, c, h, w, x, dy, gamma, beta, save_mean, save_invstd, dx, dgamma, dbeta, ws, stream=None,
                            layout=LAYOUT_NHWC):
    _check(lib().bn_bwd_batchstats_xmask(n, c, h, w, layout, _ptr(x), _ptr(dy), _ptr(gamma), _ptr(beta), _ptr(save_mean),
                                         _ptr(save_invstd), _ptr(dx), _ptr(dgamma), _ptr(dbeta), _ptr(ws), _bytes(ws), _stream(stream)))


def bn_fwd_batchstats_bf16(n, c, h, w, x, gamma, beta, eps, residual, relu, y, relu_mask, save_mean, save_invstd, ws, stream=None,
                           layout=LAYOUT_NHWC):
    _check(lib().bn_fwd_batchstats_bf16(n, c, h, w, layout, _ptr(x), _ptr(gamma), _ptr(beta), eps, _ptr(residual), int(relu), _ptr(y),
                                        _ptr(relu_mask), _ptr(save_mean), _ptr(save_invstd), _ptr(ws), _bytes(ws), _stream(stream)))


def bn_stats_scale_shift_bf16(n, c, h, w, x, gamma, beta, eps, save_mean, save_invstd, scale, shift, ws, stream=None, layout=LAYOUT_NHWC):
    _check(lib().bn_stats_scale_shift_bf16(n, c, h, w, layout, _ptr(x), _ptr(gamma), _ptr(beta), eps, _ptr(save_mean), _ptr(save_invstd),
                                           _ptr(scale), _ptr(shift), _ptr(ws), _bytes(ws), _stream(stream)))


def bn_bwd_batchstats_bf16(n, c, h, w, x, dy, dy2, y, relu_mask, gamma, beta, save_mean, save_invstd, relu, dx, dresidual, dgamma, dbeta,
                           ws, stream=None, layout=LAYOUT_NHWC):
    _check(lib().bn_bwd_batchstats_bf16(n, c, h, w, layout, _ptr(x), _ptr(dy), _ptr(dy2), _ptr(y), _ptr(relu_mask), _ptr(gamma), _ptr(beta),
                                        _ptr(save_mean), _ptr(save_invstd), int(relu), _ptr(dx), _ptr(dresidual), _ptr(dgamma),
                                        _ptr(dbeta), _ptr(ws), _bytes(ws), _stream(stream)))


def maxpool3x3s2_fwd_bf16(n, c, h, w, x, in_scale, in_shift, y, argidx, stream=None):
    _check(lib().maxpool3x3s2_fwd_bf16(n, c, h, w, _ptr(x), _ptr(in_scale), _ptr(in_shift), _ptr(y), _ptr(argidx), _stream(stream)))


def maxpool3x3s2_bwd_bf16(n, c, h, w, dy, dy2, argidx, dx, stream=None):
    _check(lib().maxpool3x3s2_bwd_bf16(n, c, h, w, _ptr(dy), _ptr(dy2), _ptr(argidx), _ptr(dx), _stream(stream)))


def avgpool_fwd_bf16(n, c, h, w, x, y, stream=None):
    _check(lib().avgpool_fwd_bf16(n, c, h, w, _ptr(x), _ptr(y), _stream(stream)))


def avgpool_bwd_bf16(n, c, h, w, dy, dx, stream=None):
    _check(lib().avgpool_bwd_bf16(n, c, h, w, _ptr(dy), _ptr(dx), _stream(stream)))


def bn_fwd_inference(n, c, h, w, x, gamma, beta, mean, invstd, residual, relu, y, ws, stream=None, layout=LAYOUT_NHWC):
    _check(lib().bn_fwd_inference(n, c, h, w, layout, _ptr(x), _ptr(gamma), _ptr(beta), _ptr(mean), _ptr(invstd), _ptr(residual),
                                  int(relu), _ptr(y), _ptr(ws), _bytes(ws), _stream(stream)))


def bn_stats_average(c, n_sets, means, invstds, eps, mean_out, invstd_out, stream=None):
    _check(lib().bn_stats_average(c, n_sets, _ptr(means), _ptr(invstds), eps, _ptr(mean_out), _ptr(invstd_out), _stream(stream)))


def bn_bwd_batchstats(n, c, h, w, x, dy, dy2, y, gamma, save_mean, save_invstd, relu, dx, dresidual, dgamma, dbeta, ws,
                      stream=None, layout=LAYOUT_NHWC):
    _check(lib().bn_bwd_batchstats(n, c, h, w, layout, _ptr(x), _ptr(dy), _ptr(dy2), _ptr(y), _ptr(gamma), _ptr(save_mean),
                                   _ptr(save_invstd), int(relu), _ptr(dx), _ptr(dresidual), _ptr(dgamma), _ptr(dbeta),
                                   _ptr(ws), _bytes(ws), _stream(stream)))


def maxpool3x3s2_fwd(n, c, h, w, x, y, argidx, stream=None):
    _check(lib().maxpool3x3s2_fwd(n, c, h, w, _ptr(x), _ptr(y), _ptr(argidx), _stream(stream)))


def maxpool3x3s2_fwd_bnrelu_input(n, c, h, w, x, in_scale, in_shift, y, argidx, stream=None):
    _check(lib().maxpool3x3s2_fwd_bnrelu_input(n, c, h, w, _ptr(x), _ptr(in_scale), _ptr(in_shift), _ptr(y), _ptr(argidx), _stream(stream)))


def maxpool3x3s2_bwd(n, c, h, w, dy, dy2, argidx, dx, stream=None):
    _check(lib().maxpool3x3s2_bwd(n, c, h, w, _ptr(dy), _ptr(dy2), _ptr(argidx), _ptr(dx), _stream(stream)))


def avgpool_fwd(n, c, h, w, x, y, stream=None):
    _check(lib().avgpool_fwd(n, c, h, w, _ptr(x), _ptr(y), _stream(stream)))


def avgpool_bwd(n, c, h, w, dy, dx, stream=None):
    _check(lib().avgpool_bwd(n, c, h, w, _ptr(dy), _ptr(dx), _stream(stream)))


def fc_fwd(n, j, k, f, w, b, y, stream=None):
    _check(lib().fc_fwd(n, j, k, _ptr(f), _ptr(w), _ptr(b), _ptr(y), _stream(stream)))


def fc_bwd(n, j, k, f, w, dy, df, dw, db, stream=None):
    _check(lib().fc_bwd(n, j, k, _ptr(f), _ptr(w), _ptr(dy), _ptr(df), _ptr(dw), _ptr(db), _stream(stream)))


def softmax_ce(n, k, logits, labels, loss, dlogits, stream=None):
    _check(lib().softmax_ce(n, k, _ptr(logits), _ptr(labels), _ptr(loss), _ptr(dlogits), _stream(stream)))


def grad_pack_fp16(count, g, out16, stream=None):
    _check(lib().grad_pack_fp16(count, _ptr(g), _ptr(out16), _stream(stream)))


def grad_unpack_fp16(count, in16, scale, g, stream=None):
    _check(lib().grad_unpack_fp16(count, _ptr(in16), scale, _ptr(g), _stream(stream)))


def opt_hparams(eta, mu1=0.9, mu2=0.99, eps=1e-8, a_sgd=1.0, a_rms=0.0, wd=0.0, g_scale=1.0):
    return OptHparams(eta, mu1, mu2, eps, a_sgd, a_rms, wd, g_scale)


def opt_update(count, theta, delta, m, g, g16, wd_mask, hp, stream=None):
    _check(lib().opt_update(count, _ptr(theta), _ptr(delta), _ptr(m), _ptr(g), _ptr(g16), _ptr(wd_mask), C.byref(hp),
                            _stream(stream)))


def rn50_alpha_sgd(epoch, center=10.0, period=5.0):
    return lib().rn50_alpha_sgd(epoch, center, period)


TRANSITION_ELU, TRANSITION_LINEAR, TRANSITION_SIGMOID, TRANSITION_SUDDEN = 0, 1, 2, 3


def rn50_alpha_sgd_transition(epoch, transition, center=10.0, period=5.0):
    return lib().rn50_alpha_sgd_transition(epoch, center, period, transition)


def rn50_alpha_rmsprop(a_sgd, eta_rmsprop=3e-4, eta_sgd=6.4):
    return lib().rn50_alpha_rmsprop(a_sgd, eta_rmsprop, eta_sgd)


def rn50_lr_base(n_workers, b_local):
    return lib().rn50_lr_base(n_workers, b_local)


def rn50_lr_slow_start(epoch, n_workers=1024, b_local=32):
    return lib().rn50_lr_slow_start(epoch, n_workers, b_local)


def rn50_recipe_hparams(epoch, n_workers=1024, b_local=32):
    hp = OptHparams()
    _check(lib().rn50_recipe_hparams(epoch, n_workers, b_local, C.byref(hp)))
    return hp


def rn50_recipe_hparams_transition(epoch, transition, n_workers=1024, b_local=32):
    hp = OptHparams()
    _check(lib().rn50_recipe_hparams_transition(epoch, n_workers, b_local, transition, C.byref(hp)))
    return hp


def rn50_param_count():
    return lib().rn50_param_count()


def rn50_param_table():
    """[(name, offset, count, dims, kind)] in flat-arena order."""
    out = []
    for i in range(lib().rn50_param_table_size()):
        name, off, cnt, dims, kind = C.c_char_p(), _sz(), _sz(), (_i * 4)(), _i()
        _check(lib().rn50_param_table(i, C.byref(name), C.byref(off), C.byref(cnt), C.byref(dims), C.byref(kind)))
        out.append((name.value.decode(), off.value, cnt.value, tuple(dims), kind.value))
    return out


def rn50_activation_bytes(batch, variant=0):
    return lib().rn50_activation_bytes(batch, variant)


class Rn50Ctx:
    """Owns the activation arena (a torch byte tensor) and the library's plan for one batch size."""

    def __init__(self, batch, variant=0, conv_dtype=DTYPE_F32, device="cuda:0"):
        nbytes = rn50_activation_bytes(batch, variant)
        if nbytes == 0:
            raise Rn50Error(EINVAL, "unsupported batch/variant")
        self.batch = batch
        self.conv_dtype = conv_dtype
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device=device)
        h = _vp()
        _check(lib().rn50_create(C.byref(h), batch, variant, conv_dtype, self.arena.data_ptr(), nbytes))
        self.handle = h

    def close(self):
        if self.handle:
            lib().rn50_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def step(self, images, labels, theta, grad, delta, m, grad16, hp, bn_eps, loss_out, stream=None):
        _check(lib().rn50_step(self.handle, _ptr(images), _ptr(labels), _ptr(theta), _ptr(grad), _ptr(delta), _ptr(m),
                               _ptr(grad16), C.byref(hp), bn_eps, _ptr(loss_out), _stream(stream)))

    def forward_backward(self, images, labels, theta, grad, bn_eps, loss_out, stream=None):
        _check(lib().rn50_forward_backward(self.handle, _ptr(images), _ptr(labels), _ptr(theta), _ptr(grad), bn_eps,
                                           _ptr(loss_out), _stream(stream)))

    def forward_eval(self, images, theta, logits_out, stream=None):
        _check(lib().rn50_forward_eval(self.handle, _ptr(images), _ptr(theta), _ptr(logits_out), _stream(stream)))

    def set_bn_stats(self, layer, mean, invstd, stream=None):
        _check(lib().rn50_set_bn_stats(self.handle, layer, _ptr(mean), _ptr(invstd), _stream(stream)))

    def filter_flip_all(self, theta, stream=None):
        _check(lib().rn50_filter_flip_all(self.handle, _ptr(theta), _stream(stream)))

    def wgrad_groups_run(self, grad, stream=None):
        n = lib().rn50_wgrad_groups_run(self.handle, _ptr(grad), _stream(stream))
        if n < 0:
            _check(n)
        return n

    def peek(self, layer, what):
        """Copy of a stored tensor of the last step as a flat torch tensor: what = 0 conv out, 1 BN out, 2 mean,
        3 invstd of conv layer `layer`; 4 pool out, 5 pool arg index (uint8), 6 features, 7 logits, 8 dlogits."""
        cnt = _sz()
        p = lib().rn50_peek(self.handle, layer, what, C.byref(cnt), _stream())
        if not p:
            raise Rn50Error(EINVAL, "bad peek request")
        off = p - self.arena.data_ptr()
        if what == 5:
            return self.arena[off:off + cnt.value].clone()
        if self.conv_dtype == DTYPE_BF16_ACT and what in (0, 1, 4):   # activations are stored as bfloat16: widened here (exact)
            return self.arena[off:off + 2 * cnt.value].view(torch.bfloat16).float()
        return self.arena[off:off + 4 * cnt.value].view(torch.float32).clone()
