"""Sweeps tile shape and split factor of the convolution kernels over the ResNet-50 layer shapes on the GPU and prints
the rows of the tuned-plan table in csrc/conv_plans.inc.  Usage: python -m paper_1711_04325_amd.tune_conv [batch] [v1|v1.5-extra|in-step|in-step-v1.5 [steps per timing [first:last row]]]

The library reads RN50_IGEMM_PLAN / RN50_WGRAD_PLAN ("bm,bn,split") as an override of its plan selection; this script
times every candidate through the public entry points and keeps the fastest.  Shapes not in the table fall back to the
library's cost model."""
import os
import sys

import torch

from . import binding as rn

IGEMM_SPLITS = (1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 12, 14, 16, 20, 24, 32)


def _geometric(lo, hi, ratio):
    out, v = [], float(lo)
    while v <= hi:
        if int(round(v)) not in out:
            out.append(int(round(v)))
        v *= ratio
    return tuple(out)


# the split fixes how many workgroups a launch has, and a launch is fastest when they fill the chip a whole number of times:
# steps of 9 % find that fit, steps of 33-50 % usually miss it
WGRAD_SPLITS = _geometric(2, 640, 1.09)


def _time(fn, reps=8):
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def resnet50_shapes(variant="v1"):
    """Unique (C, K, R, stride, pad, H) of ResNet-50, from the library's parameter table; the first block of stages 3-5
    carries its stride on the first 1x1 ("v1") or on the 3x3 ("v1.5")."""
    shapes, cur = [], 56
    for name, off, cnt, dims, kind in rn.rn50_param_table():
        if kind != 0:
            continue
        k, r, s, c = dims
        base = name[:-2]
        if base == "stem":
            sh = (c, k, r, 2, 3, 224)
        else:
            stage, block, pos = base.split(".")
            down = 2 if (block == "b0" and stage != "s2") else 1
            sa = down if variant == "v1" else 1
            if pos == "a":
                block_in = cur
                sh = (c, k, r, sa, 0, block_in)
            elif pos == "b":
                sh = (c, k, r, down // sa, 1, block_in // sa)
                cur = block_in // down
            elif pos == "c":
                sh = (c, k, r, 1, 0, cur)
            else:
                sh = (c, k, r, down, 0, block_in)
        if sh not in shapes:
            shapes.append(sh)
    return shapes


def tune(batch, shapes, candidates=None):
    dev = "cuda:0"
    rows = []
    for (c, k, r, stride, pad, h) in shapes:
        p = (h + 2 * pad - r) // stride + 1
        d = rn.conv_desc(batch, c, h, h, k, r, r, stride, pad)
        x = torch.randn((batch, h, h, c), device=dev)
        w = torch.randn((k, r, r, c), device=dev)
        y = torch.empty((batch, p, p, k), device=dev)
        dy = torch.randn_like(y)
        dx, dw = torch.empty_like(x), torch.empty_like(w)
        for op, var, splits in ((rn.OP_FWD, "RN50_IGEMM_PLAN", IGEMM_SPLITS), (rn.OP_BWD_DATA, "RN50_IGEMM_PLAN", IGEMM_SPLITS),
                                (rn.OP_BWD_WEIGHT, "RN50_WGRAD_PLAN", WGRAD_SPLITS)):
            if op == rn.OP_BWD_DATA and c == 3:
                continue  # the stem's data gradient is never computed in a training step
            def candidate(bm, bn, sp):
                os.environ[var] = "%d,%d,%d" % (bm, bn, sp)
                ws = torch.zeros(max(16, rn.rn50_conv_workspace_bytes(d, op)), dtype=torch.uint8, device=dev)
                if ws.numel() > (2 << 30):
                    return None
                return {rn.OP_FWD: lambda: rn.conv2d_fwd(d, x, w, y, ws), rn.OP_BWD_DATA: lambda: rn.conv2d_bwd_data(d, dy, w, dx, ws),
                        rn.OP_BWD_WEIGHT: lambda: rn.conv2d_bwd_weight(d, x, dy, dw, ws)}[op]

            timed = []
            for bm in (128, 64):
                for bn in (128, 64):
                    for sp in splits:
                        fn = candidate(bm, bn, sp)
                        if fn is not None:
                            timed.append((_time(fn), bm, bn, sp))
            # the fastest of many short timings is partly luck: time the five best again, longer
            timed.sort()
            best = None
            for _, bm, bn, sp in timed[:5]:
                t = _time(candidate(bm, bn, sp), reps=40)
                if best is None or t < best[0]:
                    best = (t, bm, bn, sp)
            os.environ.pop(var, None)
            if candidates is not None:  # the fastest few, for the in-step selection
                candidates[(op, batch, c, h, k, r, stride, pad)] = (best, [e for e in timed[:6] if e[0] <= 1.06 * timed[0][0]])
            t, bm, bn, sp = best
            flop = 2.0 * batch * p * p * k * c * r * r
            rows.append("    {%d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %d},  // %.1f us, %.1f TFLOP/s" %
                        (op, batch, c, h, k, r, stride, pad, bm, bn, sp, t * 1e3, flop / t / 1e9))
            print(rows[-1], flush=True)
    return rows


def tune_in_step(batch, variant, steps=60, rows=None):
    """Second pass: a plan that is fastest alone is not always fastest inside the training step, where the filter gradients
    run on a second stream beside the main chain.  Starting from the rows timed alone, each (direction, shape) tries its
    few fastest candidates in the whole step (RN50_PLAN_OVERRIDES) and keeps one only if the step gets faster by more than
    the timing noise.  Prints the final rows."""
    from . import synth
    from .arena import flat_from_dict, logical_table
    dev = "cuda:0"
    shapes = resnet50_shapes("v1.5" if variant == 1 else "v1")
    cands = {}
    tune(batch, shapes, cands)
    g = synth.rng(0)
    theta = torch.from_numpy(flat_from_dict(synth.params(g, logical_table()))).to(dev)
    images = torch.randn((batch, 224, 224, 3), device=dev)
    labels = torch.randint(0, 1000, (batch,), dtype=torch.int32, device=dev)
    grad, delta, m = torch.empty_like(theta), torch.zeros_like(theta), torch.zeros_like(theta)
    g16 = torch.empty(theta.numel(), dtype=torch.int16, device=dev)
    loss = torch.zeros(1, device=dev)
    hp = rn.opt_hparams(1e-3, 0.9, 0.99, 1e-8, 0.07, 4e-5, wd=1e-4, g_scale=1.0 / 1024)
    chosen = {key: best[1:] for key, (best, _) in cands.items()}
    # start from the rows the library already has (earlier selections), where it has them
    import re
    inc = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc", "conv_plans.inc")
    for line in open(inc):
        mm = re.match(r"\s*\{([0-9, ]+)\}", line)
        if mm:
            v = tuple(int(t) for t in mm.group(1).split(","))
            if v[:8] in chosen:
                chosen[v[:8]] = v[8:11]

    def overrides(extra=None):
        rows = dict(chosen)
        if extra:
            rows.update(extra)
        return ";".join(",".join(str(v) for v in key + plan) for key, plan in rows.items())

    def step_ms(spec):
        os.environ["RN50_PLAN_OVERRIDES"] = spec
        ctx = rn.Rn50Ctx(batch, variant=variant)   # the arena is sized for the plans in force
        run = lambda: ctx.step(images, labels, theta, grad, delta, m, g16, hp, 2e-5, loss)
        for _ in range(3):
            run()
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(steps):
                run()
            b.record()
            torch.cuda.synchronize()
            t = a.elapsed_time(b) / steps
            best = t if best is None else min(best, t)
        ctx.close()
        return best

    base = step_ms(overrides())
    print("// in-step selection starts at %.4f ms per step" % base, flush=True)
    order = sorted(cands, key=lambda key: -cands[key][0][0])
    if rows:  # a slice of the rows (longest first), so that a large batch fits several short runs: install the rows, run the next slice
        order = order[rows[0]:rows[1]]
    for key in order:
        alts = [e[1:] for e in cands[key][1] if e[1:] != chosen[key]]
        if not alts:
            continue
        print("// %s: %d candidates" % (key, len(alts[:3])), flush=True)
        base = step_ms(overrides())      # re-measured for every row: the clock drifts by more than a row is worth
        for plan in alts[:3]:
            t = step_ms(overrides({key: plan}))
            if t < base - max(0.012, 0.001 * base):
                t2, b2 = step_ms(overrides({key: plan})), step_ms(overrides())   # confirm against a fresh baseline
                if t2 < b2 - max(0.008, 0.0007 * b2):
                    print("// %s: %s -> %s, %.4f -> %.4f ms" % (key, chosen[key], plan, b2, t2), flush=True)
                    chosen[key], base = plan, t2
    final = step_ms(overrides())
    print("// in-step selection ends at %.4f ms per step" % final, flush=True)
    os.environ.pop("RN50_PLAN_OVERRIDES", None)
    for key in cands:
        print("    {%s}," % ", ".join(str(v) for v in key + chosen[key]), flush=True)


if __name__ == "__main__":
    if os.environ.get("RN50_LIB"):
        rn.LIB_PATH = os.environ["RN50_LIB"]  # tune an alternative build of the library
    # usage: tune_conv [batch] [v1|v1.5-extra]   (v1.5-extra: only the shapes that the v1.5 stride placement adds)
    if len(sys.argv) > 2 and sys.argv[2] in ("in-step", "in-step-v1.5"):
        tune_in_step(int(sys.argv[1]), 1 if sys.argv[2] == "in-step-v1.5" else 0, steps=int(sys.argv[3]) if len(sys.argv) > 3 else 60,
                     rows=tuple(int(t) for t in sys.argv[4].split(":")) if len(sys.argv) > 4 else None)
        sys.exit(0)
    v1 = resnet50_shapes("v1")
    which = sys.argv[2] if len(sys.argv) > 2 else "v1"
    tune(int(sys.argv[1]) if len(sys.argv) > 1 else 32, v1 if which == "v1" else [sh for sh in resnet50_shapes("v1.5") if sh not in v1])
