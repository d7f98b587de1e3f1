#!/usr/bin/env python3
"""Benchmark of one GPU's share of the ResNet-50 training step (the paper's per-worker minibatch of 32).

A "step" is one pass of the whole hot path over one synthetic batch resident in HBM: forward, loss, backward,
fp32->fp16 gradient pack, unpack*1/1024 and the RMSprop-warm-up update, all through rn50_step of librn50.so.
Prints ONE JSON line.  Also timed, with events on the stream the kernels run on: every convolution of the
network in the step's own launch configuration (the `roofline` object: fp32-MFMA bound), the bandwidth-bound
kernels (`kernels`), and the fp64 CPU oracle on a bounded sample of the same workload (`cpu_baseline`).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_F32 = 157.3   # TFLOP/s, dense fp32 MFMA, MI355X
PEAK_MFMA_BF16 = 2500.0  # TFLOP/s, dense bf16 MFMA
PEAK_HBM = 8000.0       # GB/s


def conv_layers(variant="v1"):
    """(name, C, K, R, stride, pad, H_in) of the 53 convolutions, from the library's own parameter table.  The block
    structure fixes resolutions and strides: stem 224 -> 112, pool -> 56; the first block of stages 3-5 halves the
    resolution, on its first 1x1 ("v1") or on its 3x3 ("v1.5"), and on its projection."""
    from paper_1711_04325_amd import binding as rn
    layers, cur = [], 56
    for name, off, cnt, dims, kind in rn.rn50_param_table():
        if kind != 0:
            continue
        base = name[:-2]
        k, r, s, c = dims
        if base == "stem":
            layers.append((base, c, k, r, 2, 3, 224))
            continue
        stage, block, pos = base.split(".")
        down = 2 if (block == "b0" and stage != "s2") else 1
        sa = down if variant == "v1" else 1
        if pos == "a":
            block_in = cur
            layers.append((base, c, k, r, sa, 0, block_in))
        elif pos == "b":
            layers.append((base, c, k, r, down // sa, 1, block_in // sa))
            cur = block_in // down
        elif pos == "c":
            layers.append((base, c, k, r, 1, 0, cur))
        else:
            layers.append((base, c, k, r, down, 0, block_in))
    return layers


def conv_bytes(batch, variant="v1"):
    """Compulsory bytes of all convolution launches of a step: x + w + y once per direction (stem: two directions)."""
    total = 0
    for name, c, k, r, stride, pad, h in conv_layers(variant):
        p = (h + 2 * pad - r) // stride + 1
        total += 4 * (batch * h * h * c + k * r * r * c + batch * p * p * k) * (2 if name == "stem" else 3)
    return total


def time_events(fn, reps, torch):
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps  # ms per call


def conv_leg(batch, torch, rn, reps=20, in_dtype=0, variant="v1"):
    """Every convolution launch of one step (fwd, bwd_weight, bwd_data except the stem's), each timed back to back, as the
    step launches them: the data gradients take filters that are already flipped (the step flips all of them in one launch,
    which the caller times once and adds)."""
    dev = "cuda:0"
    total_ms, total_flop, per_shape, wgrad_ms = 0.0, 0.0, {}, 0.0
    cache, cache_name, ceil_ms, stats_ms = {}, {}, 0.0, 0.0
    peak_tflops = PEAK_MFMA_BF16 if in_dtype else PEAK_MFMA_F32
    for name, c, k, r, stride, pad, h in conv_layers(variant):
        # the c convolution of a block applies the BN + ReLU of the b layer to its input as it loads (forward and filter gradient)
        fused = name.endswith(".c")
        key = (c, k, r, stride, h, fused)
        if key not in cache:
            p = (h + 2 * pad - r) // stride + 1
            # with bf16 activations every activation tensor is bf16 in memory, except the image in front of the first layer
            act16 = in_dtype == rn.DTYPE_BF16_ACT
            first = name == "stem"
            d = rn.conv_desc(batch, c, h, h, k, r, r, stride, pad, in_dtype=rn.DTYPE_BF16_ACT_F32IN if (act16 and first) else in_dtype)
            adt = torch.bfloat16 if act16 else torch.float32
            x = torch.randn((batch, h, h, c), device=dev).to(torch.float32 if first else adt)
            w = torch.randn((k, r, r, c), device=dev) * (2.0 / (c * r * r)) ** 0.5
            y = torch.empty((batch, p, p, k), device=dev, dtype=adt)
            dy = torch.randn((batch, p, p, k), device=dev).to(adt)
            dx, dw = torch.empty_like(x), torch.empty_like(w)
            ws = torch.zeros(max(16, max(rn.rn50_conv_workspace_bytes(d, op) for op in range(5))), dtype=torch.uint8, device=dev)
            wt = torch.empty((c, r, r, k), device=dev)
            rn.conv2d_filter_flip(d, w, wt)
            flop = 2.0 * batch * p * p * k * c * r * r
            # compulsory bytes: input (a strided 1x1 convolution touches one pixel in stride^2), filter and output once
            x_elems = batch * p * p * c if (r == 1 and stride > 1) else batch * h * h * c
            esz = 2.0 if act16 else 4.0
            nbytes = (4.0 if (first or not act16) else 2.0) * x_elems + 4.0 * k * r * r * c + esz * batch * p * p * k
            ceiling = min(peak_tflops, flop / nbytes * PEAK_HBM / 1e3)   # TFLOP/s: min(MFMA peak, flop/B x HBM peak)
            sc, sh = (torch.rand(c, device=dev) + 0.5, torch.randn(c, device=dev)) if fused else (None, None)
            if fused:
                t_f = time_events(lambda: rn.conv2d_fwd_bnrelu_input(d, x, sc, sh, w, y, ws), reps, torch)
                t_w = time_events(lambda: rn.conv2d_bwd_weight_bnrelu_input(d, x, sc, sh, dy, dw, ws), reps, torch)
            else:
                t_f = time_events(lambda: rn.conv2d_fwd(d, x, w, y, ws), reps, torch)
                t_w = time_events(lambda: rn.conv2d_bwd_weight(d, x, dy, dw, ws), reps, torch)
            # the forward call as the step makes it: the same convolution gathering the BN statistics of its output, and the
            # small kernel that merges them (where the first layer's own kernel runs: the separate statistics pass)
            ga, be = torch.ones(k, device=dev), torch.zeros(k, device=dev)
            st4 = [torch.empty(k, device=dev) for _ in range(4)]
            t_fs = time_events(lambda: rn.conv2d_fwd_bnstats(d, x, sc, sh, w, y, ga, be, 2e-5, *st4, ws), reps, torch)
            # (the first layer's data gradient is not part of a step; with bf16 activations it does not exist)
            t_d = None if (first and act16) else time_events(lambda: rn.conv2d_bwd_data_flipped(d, dy, wt, dx, ws), reps, torch)
            cache[key] = (flop, t_f, t_w, t_d, ceiling, t_fs)
            plans = {nm: "%dx%d/%d/%dwg" % rn.rn50_conv_plan(d, op) for nm, op in (("fwd", rn.OP_FWD), ("bwd_weight", rn.OP_BWD_WEIGHT),
                                                                                  ("bwd_data", rn.OP_BWD_DATA_FLIPPED))}
            per_shape["%dx%d_%d_%d_s%d_h%d%s" % (r, r, c, k, stride, h, "_bnrelu_input" if fused else "")] = {
                "gflop": round(flop / 1e9, 3), "layers": 0, "min_MB": round(nbytes / 1e6, 1), "ceiling_tflops": round(ceiling, 1),
                "bound": "hbm" if ceiling < peak_tflops else "mfma",
                "fwd_tflops": round(flop / t_f / 1e9, 1), "bwd_weight_tflops": round(flop / t_w / 1e9, 1),
                "bwd_data_tflops": round(flop / t_d / 1e9, 1) if t_d else None,
                "fwd_us": round(t_f * 1e3, 1), "fwd_with_bn_statistics_us": round(t_fs * 1e3, 1), "bwd_weight_us": round(t_w * 1e3, 1), "bwd_data_us": round(t_d * 1e3, 1) if t_d else None,
                "frac_of_shape_ceiling": {"fwd": round(flop / t_f / 1e9 / ceiling, 3), "bwd_weight": round(flop / t_w / 1e9 / ceiling, 3),
                                          "bwd_data": round(flop / t_d / 1e9 / ceiling, 3) if t_d else None},
                "plan(tile/split/workgroups)": plans}
            cache_name[key] = "%dx%d_%d_%d_s%d_h%d%s" % (r, r, c, k, stride, h, "_bnrelu_input" if fused else "")
            del x, w, y, dy, dx, dw, ws, wt
        flop, t_f, t_w, t_d, ceiling, t_fs = cache[key]
        stats_ms += t_fs - t_f
        per_shape[cache_name[key]]["layers"] += 1
        ndir = 2 if name == "stem" else 3   # the stem's data gradient is never needed
        ceil_ms += ndir * flop / ceiling / 1e9
        total_ms += t_f + t_w + (0.0 if name == "stem" else t_d)
        wgrad_ms += 0.0 if name == "stem" else t_w    # what a context with grouped filter gradients launches differently
        total_flop += ndir * flop
    return total_ms, total_flop, per_shape, ceil_ms, stats_ms, wgrad_ms


def measured_ceilings(torch, rn, bf16=False):
    """What the machine sustains on kernels of known work (library probes, timed with events on their stream): a loop of
    nothing but MFMAs, and a plain 1 GiB copy.  Context for the data-sheet peaks the fractions are quoted against."""
    dev = "cuda:0"
    out = {}
    sink = torch.empty(65536 * 2, device=dev)
    ticks = torch.zeros(2, dtype=torch.int64, device=dev)

    def mhz():
        c, w = (int(v) for v in ticks.cpu())
        return round(100.0 * c / w, 0) if w else None

    for tag, dt, iters in (("mfma_f32_tflops", rn.DTYPE_F32, 4000),) + ((("mfma_bf16_tflops", rn.DTYPE_BF16, 16000),) if bf16 else ()):
        flop = rn.rn50_probe_mfma(dt, iters, 2, sink)          # warm-up (and the clock settles under load)
        t = time_events(lambda: rn.rn50_probe_mfma(dt, iters, 2, sink, ticks), 5, torch)
        out[tag] = round(flop / t / 1e9, 1)
        out[tag.replace("_tflops", "_shader_mhz")] = mhz()
    # the same loop cut to the length of a layer's launch (the convolutions of this workload take 20-160 us each): the clock
    # of a short kernel stays below the sustained one, so a layer-sized launch of nothing but MFMAs does not reach the long
    # loop's rate either
    out["mfma_f32_layer_sized"] = []
    for iters in (14, 56):
        flop = rn.rn50_probe_mfma(rn.DTYPE_F32, iters, 2, sink)
        t = time_events(lambda: rn.rn50_probe_mfma(rn.DTYPE_F32, iters, 2, sink, ticks), 50, torch)
        out["mfma_f32_layer_sized"].append({"us_per_launch": round(t * 1e3, 1), "tflops": round(flop / t / 1e9, 1), "shader_mhz": mhz()})
    n = 256 << 20                                              # 1 GiB in, 1 GiB out: far larger than every cache
    src, dst = torch.ones(n, device=dev), torch.empty(n, device=dev)
    t = time_events(lambda: rn.rn50_probe_copy(n, src, dst), 10, torch)
    out["hbm_copy_GBps"] = round(8.0 * n / t / 1e6, 1)
    t = time_events(lambda: rn.rn50_probe_empty(256, 2000), 3, torch) / 2000
    out["empty_launch_us"] = round(t * 1e3, 2)     # back to back on one stream, enqueued by one call: the floor of a dependent launch
    out["how"] = "rn50_probe_mfma (512 workgroups x 4 wavefronts of back-to-back MFMAs, about 5 ms per launch; layer_sized: the same loop at 448 and 1792 MFMAs per wavefront, 50 launches back to back; shader_mhz from the kernel's own cycle and 100 MHz reference counters), rn50_probe_copy (1 GiB read + 1 GiB written), rn50_probe_empty (2000 launches of 256 idle workgroups)"
    return out


def bn_family_leg(batch, torch, rn, variant="v1", reps=5, stats_in_conv_ms=None):
    """Every BN call of one training step, forward then backward, in the form the step uses for its layer, each on its own
    tensors (1.4 GB of convolution outputs at batch 32, so nothing is served from a cache across repetitions), enqueued back to
    back on one stream and timed as a whole with events.  Forward: the statistics come out of the convolutions (their cost is
    stats_in_conv_ms, measured by the convolution pass), so what is left is the normalising pass where the consumer does not
    normalise as it loads (byte mask for the residual-carrying layers), and the first layer's separate statistics pass.
    Backward: mask rebuilt from the input where there is no residual.  Bytes are algorithmic bytes of these passes (each
    tensor a pass must read or write counted once per pass)."""
    dev = "cuda:0"
    layers = []
    for name, c, k, r, stride, pad, h in conv_layers(variant):
        p = (h + 2 * pad - r) // stride + 1
        pos = "stem" if name == "stem" else name.rsplit(".", 1)[1]
        layers.append((pos, k, p))
    big = max(batch * p * p * k for _, k, p in layers)
    bufs = [torch.randn(big, device=dev) for _ in range(4)]     # incoming gradient, second gradient / residual, outgoing gradient, shortcut gradient
    wsb = torch.zeros(max(rn.rn50_bn_workspace_bytes(batch, k, p, p) for _, k, p in layers), dtype=torch.uint8, device=dev)
    calls, nbytes_f, nbytes_b, nfwd = [], 0.0, 0.0, 0
    last_c = max(i for i, l in enumerate(layers) if l[0] == "c")
    for i, (pos, k, p) in enumerate(layers):
        e = batch * p * p * k
        x = torch.randn(e, device=dev)
        ga, be = torch.ones(k, device=dev), torch.zeros(k, device=dev)
        mean, inv, sc, sh, dg, db = (torch.empty(k, device=dev) for _ in range(6))
        a = (batch, k, p, p)
        sc.fill_(1.0)
        sh.zero_()
        mean.zero_()
        inv.fill_(1.0)
        if pos == "stem":             # its own convolution kernel gathers nothing: the separate statistics pass
            fwd = (lambda a=a, x=x, ga=ga, be=be, mean=mean, inv=inv, sc=sc, sh=sh: rn.bn_stats_scale_shift(*a, x, ga, be, 2e-5, mean, inv, sc, sh, wsb))
            nbytes_f += 4.0 * e
            nfwd += 2
        elif pos == "b":              # statistics from the convolution, normalised by the consumer: nothing to do
            fwd = (lambda: None)
        elif pos == "c":
            y, mask = torch.empty(e, device=dev), torch.empty(e // 4, dtype=torch.uint8, device=dev)
            fwd = (lambda a=a, x=x, sc=sc, sh=sh, y=y, mask=mask: rn.bn_fwd_apply(*a, x, sc, sh, bufs[1], 1, y, mask))
            nbytes_f += 12.25 * e
            nfwd += 1
        else:                         # a: BN + ReLU written; p: BN written
            y = torch.empty(e, device=dev)
            fwd = (lambda a=a, x=x, sc=sc, sh=sh, y=y, relu=int(pos == "a"): rn.bn_fwd_apply(*a, x, sc, sh, None, relu, y))
            nbytes_f += 8.0 * e
            nfwd += 1
        if pos == "c":
            dy2 = None if i == last_c else bufs[1]
            bwd = (lambda a=a, x=x, mask=mask, ga=ga, mean=mean, inv=inv, dg=dg, db=db, dy2=dy2:
                   rn.bn_bwd_batchstats_mask(*a, x, bufs[0], dy2, mask, ga, mean, inv, bufs[2], bufs[3], dg, db, wsb))
            nbytes_b += (24.25 if dy2 is None else 28.25) * e
        elif pos == "p":
            bwd = (lambda a=a, x=x, ga=ga, mean=mean, inv=inv, dg=dg, db=db: rn.bn_bwd_batchstats(*a, x, bufs[0], None, None, ga, mean, inv, 0, bufs[2], None, dg, db, wsb))
            nbytes_b += 20.0 * e
        else:
            bwd = (lambda a=a, x=x, ga=ga, be=be, mean=mean, inv=inv, dg=dg, db=db: rn.bn_bwd_batchstats_xmask(*a, x, bufs[0], ga, be, mean, inv, bufs[2], dg, db, wsb))
            nbytes_b += 20.0 * e
        calls.append((fwd, bwd))

    def one_pass():
        for fwd, _ in calls:
            fwd()
        for _, bwd in reversed(calls):
            bwd()
    ms = time_events(one_pass, reps, torch)
    total = nbytes_f + nbytes_b
    out = {"ms_per_step": round(ms, 4), "algorithmic_bytes": total, "GBps": round(total / ms / 1e6, 1),
           "frac_of_hbm_peak": round(total / ms / 1e6 / PEAK_HBM, 4), "launches": nfwd + 3 * len(calls),
           "what": "the BN passes of one step that are kernels of their own (forward: normalising passes and the first layer's "
                   "statistics; backward: all %d layers), each on its own tensors, back to back on one stream" % len(calls)}
    if stats_in_conv_ms is not None:
        # the statistics gathered inside the forward convolutions read and write no tensor of their own: time, no bytes
        out["with_statistics_in_conv"] = {"ms_per_step": round(ms + stats_in_conv_ms, 4), "GBps": round(total / (ms + stats_in_conv_ms) / 1e6, 1),
                                          "frac_of_hbm_peak": round(total / (ms + stats_in_conv_ms) / 1e6 / PEAK_HBM, 4)}
    return out


def tracked_traffic(batch, bf16, variant):
    """HBM bytes of all convolution launches of one step from rocprofv3 counter runs (FETCH_SIZE, WRITE_SIZE, scaled by a copy
    of known size): taken from the tracked summary profiles/rn50_step_n32_hbm_traffic.json and only when that summary was
    measured on the kernel sources this run uses; otherwise null.  This run does not measure it."""
    path = os.path.join(ROOT, "profiles", "rn50_step_n32_hbm_traffic.json")
    if batch != 32 or bf16 or variant != "v1" or not os.path.exists(path):
        return None, None
    rec = json.load(open(path))
    if rec.get("kernel_source_sha256") != kernel_source_hash():
        return None, "profiles/rn50_step_n32_hbm_traffic.json is stale (measured on other kernel sources)"
    return rec["conv_family_bytes_per_step"], "profiles/rn50_step_n32_hbm_traffic.json (commit %s)" % rec.get("commit", "?")


def kernel_source_hash():
    """sha256 over the sources the convolution launches are built from, in name order."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_1711_04325_amd", "csrc")
    for f in ("common.h", "conv.hip", "conv_kernels.h", "conv_plans.inc", "conv_plans_bf16act.inc"):
        h.update(f.encode())
        h.update(open(os.path.join(csrc, f), "rb").read())
    return h.hexdigest()


def bandwidth_leg(batch, torch, rn, reps=10):
    """Achieved HBM GB/s (algorithmic bytes) of the bandwidth-bound kernels at the step's largest shapes."""
    dev = "cuda:0"
    out = {}
    n = rn.rn50_param_count()
    g = torch.randn(n, device=dev)
    g16 = torch.empty(n, dtype=torch.int16, device=dev)
    th, de, m = torch.randn(n, device=dev), torch.zeros(n, device=dev), torch.zeros(n, device=dev)
    hp = rn.opt_hparams(6.4, 0.9, 0.99, 1e-8, 0.07, 4e-5, wd=1e-4, g_scale=1.0 / 1024)
    t = time_events(lambda: rn.grad_pack_fp16(n, g, g16), reps, torch)
    out["grad_pack_fp16"] = {"ms": round(t, 4), "GBps": round(6.0 * n / t / 1e6, 1), "bytes_per_elem": 6}
    t = time_events(lambda: rn.opt_update(n, th, de, m, None, g16, None, hp), reps, torch)
    out["opt_update_fp16"] = {"ms": round(t, 4), "GBps": round(26.0 * n / t / 1e6, 1), "bytes_per_elem": 26}
    for (c, h) in ((64, 112), (256, 56), (512, 28), (1024, 14), (2048, 7)):
        x = torch.randn((batch, h, h, c), device=dev)
        y, dy, dx = torch.empty_like(x), torch.randn_like(x), torch.empty_like(x)
        ga, be = torch.ones(c, device=dev), torch.zeros(c, device=dev)
        mean, inv, dg, db = (torch.empty(c, device=dev) for _ in range(4))
        ws = torch.zeros(rn.rn50_bn_workspace_bytes(batch, c, h, h), dtype=torch.uint8, device=dev)
        elems = x.numel()
        t = time_events(lambda: rn.bn_fwd_batchstats(batch, c, h, h, x, ga, be, 2e-5, None, 1, y, mean, inv, ws), reps, torch)
        out["bn_fwd_relu_%dx%d" % (c, h)] = {"ms": round(t, 4), "GBps": round(12.0 * elems / t / 1e6, 1), "bytes_per_elem": 12}
        t = time_events(lambda: rn.bn_bwd_batchstats(batch, c, h, h, x, dy, None, y, ga, mean, inv, 1, dx, None, dg, db, ws), reps, torch)
        out["bn_bwd_relu_%dx%d" % (c, h)] = {"ms": round(t, 4), "GBps": round(28.0 * elems / t / 1e6, 1), "bytes_per_elem": 28}
    return out


def cpu_baseline(sample_batch, variant="v1"):
    """The fp64 oracle, as it stands, on a bounded sample (a smaller batch of the same 3x224x224 workload)."""
    import numpy as np
    from oracle import ops as orc
    from oracle import resnet50
    from paper_1711_04325_amd import synth
    g = synth.rng(0)
    images = synth.normal(g, (sample_batch, 3, 224, 224))
    params = {k: v.astype(np.float64) for k, v in synth.params(g, resnet50.param_table()).items()}
    labels = synth.labels(g, sample_batch)
    t0 = time.time()
    loss, grads = resnet50.forward_backward(params, images, labels, variant=variant)
    flat = resnet50.flatten(grads).astype(np.float32)
    z = np.zeros(flat.size)
    resnet50.communicate_and_update(resnet50.flatten(params), z, z, flat, dict(eta=6.4, mu1=0.9, mu2=0.99, eps=1e-8, a_sgd=0.07,
                                                                                a_rms=4e-5, wd=1e-4))
    dt = time.time() - t0
    return {"value": round(sample_batch / dt, 3), "unit": "images/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": "one full training step (fwd+bwd+pack+update) at batch %d of the same 3x224x224 workload, %.1f s" % (sample_batch, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--conv-dtype", choices=("f32", "bf16", "bf16act"), default="f32",
                    help="operand precision of the convolutions (f32 is the paper's and the headline; bf16 rounds operands "
                         "on the way into LDS; bf16act also keeps every activation and activation gradient as bf16 in memory; "
                         "both are reported under their own metric names)")
    ap.add_argument("--variant", choices=("v1", "v1.5"), default="v1",
                    help="where the stride of a stage's first block sits: on its first 1x1 (v1, the headline) or its 3x3")
    ap.add_argument("--cpu-sample-batch", type=int, default=32)
    ap.add_argument("--no-legs", action="store_true", help="skip the per-kernel and CPU legs (profiling runs)")
    ap.add_argument("--no-side-stream", action="store_true",
                    help="run the filter gradients on the caller's stream instead of the context's helper stream, so that a "
                         "profiler sees every kernel's duration without another kernel sharing the chip")
    ap.add_argument("--wgrad-group", type=int, default=None, 
                    help="filter gradients per layer (0) or in grouped launches of this many blocks each (16: all at once); default: the library's")
    ap.add_argument("--wgrad-group-wgs-per-cu", type=int, default=None, help="grouped filter gradients: workgroups per CU at most (0: what fits)")
    ap.add_argument("--wgrad-group-stages", type=int, default=None, help="grouped filter gradients: LDS stages per work item")
    ap.add_argument("--wgrad-group-tile", default=None, help="grouped filter gradients: tile, e.g. 64,64")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time its replays instead of eager launches (same kernels, same results; "
                         "the hyperparameters are those of the captured call)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="run three 256 MiB copies (rn50_probe_copy) first: a kernel of known traffic to scale HBM byte counters with")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on one GPU only (the all-reduce between workers is not part of it); use --gpus 1")

    import torch
    from paper_1711_04325_amd import binding as rn
    if a.no_side_stream:
        rn.rn50_set_option("side_stream", "0")
    for opt, val in (("wgrad_group", a.wgrad_group), ("wgrad_group_stages", a.wgrad_group_stages), ("wgrad_group_tile", a.wgrad_group_tile),
                     ("wgrad_group_wgs_per_cu", a.wgrad_group_wgs_per_cu)):
        if val is not None:
            rn.rn50_set_option(opt, val)
    from paper_1711_04325_amd import synth
    from paper_1711_04325_amd.arena import flat_from_dict, logical_table

    dev = "cuda:0"
    torch.cuda.set_device(0)
    batch = a.batch
    g = synth.rng(0)
    images = synth.normal(g, (batch, 3, 224, 224))
    params = synth.params(g, logical_table())
    labels = synth.labels(g, batch)
    dimg = torch.from_numpy(images.transpose(0, 2, 3, 1).copy()).to(dev)
    dlab = torch.from_numpy(labels).to(dev)
    theta = torch.from_numpy(flat_from_dict(params)).to(dev)
    count = theta.numel()
    grad, delta, m = torch.empty_like(theta), torch.zeros_like(theta), torch.zeros_like(theta)
    g16 = torch.empty(count, dtype=torch.int16, device=dev)
    loss = torch.zeros(1, device=dev)
    bf16 = a.conv_dtype != "f32"
    act16 = a.conv_dtype == "bf16act"
    ctx = rn.Rn50Ctx(batch, variant=rn.VARIANT_V15 if a.variant == "v1.5" else rn.VARIANT_V1,
                     conv_dtype=rn.DTYPE_BF16_ACT if act16 else rn.DTYPE_BF16 if bf16 else rn.DTYPE_F32)
    # a blend point of the warm-up (epoch 5): both the SGD and the RMSprop term are active; 1/1024 = 1/#workers
    eta = 1e-3  # small enough that 50+ steps on one fixed batch stay finite; the arithmetic per step is unchanged
    a_sgd = rn.rn50_alpha_sgd(5.0)
    hp = rn.opt_hparams(eta, 0.9, 0.99, 1e-8, a_sgd, rn.rn50_alpha_rmsprop(a_sgd, 3e-4, 6.4), wd=1e-4, g_scale=1.0 / 1024)

    def step():
        ctx.step(dimg, dlab, theta, grad, delta, m, g16, hp, 2e-5, loss)

    if a.calib_copy:
        src = torch.zeros(64 << 20, device=dev)          # 256 MiB of fp32
        dst = torch.empty_like(src)
        for _ in range(3):
            rn.rn50_probe_copy(src.numel(), src, dst)     # probe_copy_kernel: 256 MiB read, 256 MiB written per dispatch
        torch.cuda.synchronize()
    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    if a.graph:
        cap = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=cap):
            ctx.step(dimg, dlab, theta, grad, delta, m, g16, hp, 2e-5, loss, stream=torch.cuda.current_stream().cuda_stream)
        step = graph.replay
        step()
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.time()
    e0.record()
    for _ in range(a.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.time() - t0) * 1e3 / a.steps
    ms = e0.elapsed_time(e1) / a.steps
    ms = max(ms, wall_ms)
    final_loss = loss.item()
    if not (final_loss == final_loss and abs(final_loss) < 1e6):
        sys.exit("bench.py: the loss is not finite (%r)" % final_loss)

    out = {"metric": "resnet50%s_train_images_per_s_1gpu_bs%d%s" % ("" if a.variant == "v1" else "_v1.5", batch, "_bf16act" if act16 else "_bf16conv" if bf16 else ""), "value": round(batch / ms * 1e3, 1), "unit": "images/s",
           "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
           "config": {"workload": "full ResNet-50 " + a.variant + " training step at the paper's per-worker minibatch: %d synthetic 3x224x224 "
                                  "images, 1000 classes, BN with batch statistics only, fwd+bwd, fp32->fp16 gradient pack, "
                                  "unpack*1/1024, RMSprop-warm-up update (alpha_SGD of epoch 5)" % batch,
                      "global_batch": batch, "params": count, "launch": "graph replay" if a.graph else "eager"},
           "final_loss": round(final_loss, 5)}
    if not a.no_legs:
        conv_ms, conv_flop, per_shape, ceil_ms, stats_ms, wgrad_layer_ms = conv_leg(batch, torch, rn, variant=a.variant,
                                                          in_dtype=rn.DTYPE_BF16_ACT if act16 else rn.DTYPE_BF16 if bf16 else rn.DTYPE_F32)
        flip_ms = time_events(lambda: ctx.filter_flip_all(theta), 20, torch)   # the step's one launch that flips every filter
        conv_ms += flip_ms
        # a context that launches its filter gradients in groups: those launches as the step makes them (back to back on the
        # buffers the last step left) in place of the per-layer calls timed above
        ngroups = ctx.wgrad_groups_run(grad)
        grouped_ms = time_events(lambda: ctx.wgrad_groups_run(grad), 10, torch) if ngroups else None
        if ngroups:
            conv_ms += grouped_ms - wgrad_layer_ms
        ach = conv_flop / conv_ms / 1e9
        peak = PEAK_MFMA_BF16 if bf16 else PEAK_MFMA_F32
        # Not the step's schedule unless the context groups: the same filter gradients as ONE grouped launch (conv2d_bwd_weight_group
        # through a second context created with wgrad_group = 16, on the buffers one pass of it leaves), alone on the chip.
        alt = None
        if not ngroups and not bf16:
            rn.rn50_set_option("wgrad_group", "16")
            try:
                ctx2 = rn.Rn50Ctx(batch, variant=rn.VARIANT_V15 if a.variant == "v1.5" else rn.VARIANT_V1)
            finally:
                rn.rn50_set_option("wgrad_group", None if a.wgrad_group is None else a.wgrad_group)
            ctx2.forward_backward(dimg, dlab, theta, grad, 2e-5, loss)
            torch.cuda.synchronize()
            g_ms = time_events(lambda: ctx2.wgrad_groups_run(grad), 10, torch)
            alt_ms = conv_ms - wgrad_layer_ms + g_ms
            alt = {"filter_gradients_ms_per_step": round(g_ms, 4), "conv_ms_per_step": round(alt_ms, 4),
                   "achieved": round(conv_flop / alt_ms / 1e9, 2), "frac": round(conv_flop / alt_ms / 1e9 / peak, 4),
                   "what": "the convolution family with the 52 filter gradients behind the first layer in one grouped launch, timed alone; "
                           "the step does not launch them this way by default (inside the two-stream step the grouped launch is slower)"}
            ctx2.close()
            del ctx2
        ceilings = measured_ceilings(torch, rn, bf16)
        traffic, traffic_source = tracked_traffic(batch, bf16, a.variant)
        meas = ceilings["mfma_bf16_tflops" if bf16 else "mfma_f32_tflops"]
        out["roofline"] = {"bound": "mfma", "achieved": round(ach, 2), "peak": peak, "unit": "TFLOP/s",
                           "frac": round(ach / peak, 4),
                           "traffic": traffic, "traffic_source": traffic_source,
                           "algorithmic_bytes": conv_bytes(batch, a.variant) if not act16 else None,
                           "peak_measured": ceilings, "frac_of_measured_mfma": round(ach / meas, 4),
                           # every layer at its own ceiling min(MFMA peak, flop/byte x HBM peak) would take ceiling_ms_per_step
                           "ceiling_ms_per_step": round(ceil_ms, 4), "frac_of_shape_ceilings": round(ceil_ms / (conv_ms - flip_ms), 4),
                           "kernel": "igemm_kernel / wgrad_kernel (%s MFMA implicit-GEMM convolutions): all 158 convolution "
                                     "launches of one step and its one filter-flip launch, each timed with events on its stream" % a.conv_dtype,
                           "flop_per_step": conv_flop, "ms_per_step": round(conv_ms, 4),
                           "with_grouped_filter_gradients": alt,
                           "filter_gradients": {"launches_per_step": (ngroups + 1) if ngroups else 53,
                                                "grouped_ms_per_step": round(grouped_ms, 4) if ngroups else None,
                                                "layer_by_layer_ms_per_step": round(wgrad_layer_ms, 4),
                                                "what": "every filter gradient behind the first layer's: in the step's grouped launches "
                                                        "(counted in ms_per_step when the context groups) and as one call per layer"},
                           # what the step's forward calls add to these launches: the BN statistics gathered as the output
                           # tiles are written and the kernel that merges them (conv2d_fwd_bnstats against conv2d_fwd)
                           "bn_statistics_in_forward_ms_per_step": round(stats_ms, 4)}
        out["conv_fraction_of_step"] = round(conv_ms / ms, 3)
        out["conv_shapes"] = per_shape
        out["kernels"] = bandwidth_leg(batch, torch, rn)
        if not act16:     # the BN-family pass below times the fp32-storage calls
          out["bandwidth"] = {"bound": "hbm", "peak": PEAK_HBM, "unit": "GB/s", "peak_measured_copy": ceilings["hbm_copy_GBps"],
                            "bn_family": bn_family_leg(batch, torch, rn, a.variant, stats_in_conv_ms=stats_ms),
                            "grad_pack_fp16": out["kernels"]["grad_pack_fp16"], "opt_update_fp16": out["kernels"]["opt_update_fp16"]}
        out["cpu_baseline"] = cpu_baseline(a.cpu_sample_batch, a.variant)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
