#!/usr/bin/env python3
"""Benchmark: operator evaluation throughput (forward + backward) on one MI355X.

A step is one training-step evaluation of the conv-equivalent synthesized operator (Unfold 3x3, Share, Reduce over
C,kh,kw) at the four ResNet-18 stage shapes with N=32: forward, backward-data and backward-weight of every shape,
twelve library calls.  The step is timed once per input type and the two are never blended: the headline `value`
is the fp32 step (the paper's precision), the bf16-input step is reported next to it under "bf16" with its own
roofline block.  Inputs are synthetic, seeded, resident in HBM before the timed region, and rotate over several
buffer sets so that launches read HBM and not the last-level cache.  The other workloads (grouped shift-unfold
forward and training step, strided depthwise, Operator 1, the QKV matrix product, pure views) are timed per call
under "detail".  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}

def alg_bytes(w, which, in_bytes, out_bytes):
    """Algorithmic traffic of one call: each operand read once, the result written once."""
    import numpy as np
    nx, nw, no = (int(np.prod(s)) for s in (w.x_shape, w.w_shape, w.out_shape))
    if which == 0:
        return (nx + nw) * in_bytes + no * out_bytes
    if which == 1:
        return (no + nw) * in_bytes + nx * out_bytes
    return (nx + no) * in_bytes + nw * 4


def stored_profile(kind, family):
    """A figure from a committed rocprofv3 summary (profiles/<kind>_<family>.txt, `key: value` lines), valid only
    while the kernel sources it was taken on are unchanged (sha256 of their concatenation)."""
    try:
        rec = {}
        for line in open(os.path.join(ROOT, "profiles", f"{kind}_{family}.txt")):
            key, sep, val = line.partition(":")
            if sep and key.strip() in ("value", "sources", "sha256"):
                rec[key.strip()] = val.split("(")[0].strip()
        srcs = [os.path.join(ROOT, "paper_2410_23745_amd", "csrc", f) for f in rec["sources"].split()]
        digest = hashlib.sha256(b"".join(open(f, "rb").read() for f in srcs)).hexdigest()
        return float(rec["value"]) if digest == rec["sha256"] else None
    except (OSError, KeyError, ValueError):
        return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--dtype", choices=("f32", "bf16", "both"), default="both",
                    help="input type of the timed step (both: fp32 is the headline, bf16 reported beside it)")
    ap.add_argument("--rotate-mb", type=float, default=600.0, help="bytes of rotating buffer sets per call")
    ap.add_argument("--config", type=int, default=-1, help="detail only for this BASELINE config (0..4); -1: all")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-detail", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: the library has no multi-GPU, collective or rank code "
              "(--gpus must be 1)", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2410_23745_amd as syno
    from syno_inputs import BF16, F32, workloads as wl
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from util import to_dev

    if not os.path.exists(syno.library_path()):
        from paper_2410_23745_amd import build
        build.build()
    syno.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    def n_sets(nbytes, cap=24):
        return int(max(2, min(cap, -(-args.rotate_mb * 1e6 // nbytes))))

    class Case:
        """One operator call with its device buffers, rotating over several sets, launches pre-bound."""

        def __init__(self, name, w, which, sets=None, plan=None):
            self.name, self.w, self.which = name, w, which
            self.plan = plan or syno.Plan(w.desc)
            inb = 2 if w.desc.in_dtype == BF16 else 4
            outb = 2 if (w.desc.out_dtype == BF16 and which != 2) else 4
            self.bytes = alg_bytes(w, which, inb, outb)
            self.flops = w.flops
            self.dtype = "bf16" if w.desc.in_dtype == BF16 else "f32"
            X, W = to_dev(w.X, w.X_bits), to_dev(w.W, w.W_bits)
            G = to_dev(w.G, w.G_bits) if w.G is not None else None
            a, b = ((X, W), (G, W), (X, G))[which]
            out_shape = (w.out_shape, w.x_shape, w.w_shape)[which]
            out_dtype = torch.float32 if which == 2 else self.plan.out_dtype
            self.n_sets = sets or n_sets(self.bytes)
            self.bufs = [(a.clone(), b.clone(), torch.empty(out_shape, dtype=out_dtype, device=dev))
                         for _ in range(self.n_sets)]
            self.calls = [self.plan.bind(which, *s) for s in self.bufs]
            self.kernel = self.plan.kernel(which)
            self.i = 0
            peak = MFMA_PEAK_TFLOPS[self.dtype]
            self.roof_tf = min(peak, self.flops / self.bytes * HBM_PEAK_GBS / 1e3)
            self.bound = "hbm" if self.roof_tf < peak else "mfma"

        def launch(self):
            self.calls[self.i % self.n_sets]()
            self.i += 1

        def launch_hot(self):
            self.calls[0]()

        def time_us(self, iters, warm=10, hot=False, reps=5):
            """Microseconds per launch: `iters` launches back to back between two events; median and mean of `reps`."""
            fn = self.launch_hot if hot else self.launch
            for _ in range(warm):
                fn()
            torch.cuda.synchronize()
            t = []
            for _ in range(reps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                for i in range(iters):
                    fn()
                b.record()
                torch.cuda.synchronize()
                t.append(a.elapsed_time(b) * 1e3 / iters)
            t.sort()
            return t[len(t) // 2], sum(t) / len(t)

        def row(self, us):
            tf = self.flops / (us * 1e-6) / 1e12
            return {"case": self.name, "kernel": self.kernel, "launch": self.plan.describe(self.which), "us": us,
                    "TFLOP/s": tf, "GB/s": self.bytes / (us * 1e-6) / 1e9, "bound": self.bound,
                    "roofline_frac": tf / self.roof_tf, "rotating_sets": self.n_sets}

    PASS = ("fwd", "bwd_data", "bwd_weight")

    def run_step(bf16):
        """Times the training step of configs[1] in one input type.  Returns the JSON fields of that step."""
        tag = "bf16" if bf16 else "f32"
        cases = []
        for stage, (C, H) in enumerate(wl.RESNET18_STAGES):
            w = wl.config1_train(stage, bf16)
            plan = syno.Plan(w.desc)
            for which in range(3):
                cases.append(Case(f"conv3x3_C{C}_{H}x{H}_N32_{tag}_{PASS[which]}", w, which, plan=plan))
        flop = sum(c.flops for c in cases)
        for _ in range(args.warmup):
            for c in cases:
                c.launch()
        torch.cuda.synchronize()
        # the timed region: K steps back to back, bracketed by a synchronisation and an event on either side (events
        # go to torch's current stream, which is the stream the binding launches on)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for k in range(args.steps):
            for c in cases:
                c.launch()
        e1.record()
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
        ms_per_step_events = e0.elapsed_time(e1) / args.steps
        # per call: the same launches again, K of one call back to back between two events (an event after every
        # single launch would add a marker and a drain of the queue per launch, several microseconds each)
        us = {}
        for c in cases:
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for k in range(max(args.steps, 10)):
                c.launch()
            b.record()
            torch.cuda.synchronize()
            us[c.name] = a.elapsed_time(b) * 1e3 / max(args.steps, 10)
        # dominant kernel = the (kernel family, pass kind) with the largest summed duration; forward and backward-data
        # run the same contraction kernel, backward-weight has its own
        groups = {}
        for c in cases:
            groups.setdefault((c.kernel, "weight_gradient" if c.which == 2 else "contraction"), []).append(c)
        key = max(groups, key=lambda g: sum(us[c.name] for c in groups[g]))
        dom = groups[key]
        # per launch: algorithmic flops (or bytes) of the call / its average duration, averaged over the group's launches
        dom_us = sum(us[c.name] for c in dom) / len(dom)
        dom_flops = sum(c.flops for c in dom) / len(dom)
        dom_bytes = sum(c.bytes for c in dom) / len(dom)
        peak = MFMA_PEAK_TFLOPS[tag]
        if dom_flops / dom_bytes * HBM_PEAK_GBS / 1e3 < peak:
            ach = dom_bytes / (dom_us * 1e-6) / 1e9
            roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS}
        else:
            ach = dom_flops / (dom_us * 1e-6) / 1e12
            roof = {"bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak}
        family = f"{key[0]}_{key[1]}"
        roof.update({"kernel": f"{key[0]}[{tag}] {key[1]}", "avg_launch_us": dom_us,
                     "launches_averaged": [c.name for c in dom],
                     "clock": "HIP events on the launch stream around K back-to-back launches of each call of the timed step "
                              "(the interval of a backward call includes its small weight-transposition / partial-sum "
                              "kernels)"})
        # the clock the dominant kernel actually runs at: its workgroups leave the constant 100 MHz counter and the shader
        # clock counter on entry and exit (an option of the plan); a launch of each call, after warm-up launches
        probe = torch.zeros(4 * 8192, dtype=torch.int64, device=dev)
        ghz = []
        if key[0].startswith("mfma_contraction"):
            for c in dom:
                probed = syno.Plan(c.w.desc, clock_probe=probe.data_ptr())
                call = probed.bind(c.which, *c.bufs[0])
                for _ in range(5):
                    call()
                torch.cuda.synchronize()
                probe.zero_()
                torch.cuda.synchronize()
                call()
                torch.cuda.synchronize()
                t = probe.view(-1, 4).cpu().numpy().astype(np.float64)
                t = t[(t[:, 0] > 0) & (t[:, 2] > t[:, 0])]
                if len(t):
                    ghz.append(float(np.median((t[:, 3] - t[:, 1]) / (t[:, 2] - t[:, 0]))) / 10.0)
        if ghz:
            clock = sum(ghz) / len(ghz)
            roof.update({"sustained_clock_GHz": clock, "nominal_clock_GHz": 2.4,
                         "frac_of_peak_at_sustained_clock": roof["frac"] * 2.4 / clock,
                         "sustained_clock_note": "median over workgroups of (shader-clock ticks) / (100 MHz ticks) between a "
                                                 "workgroup's entry and exit, mean over the averaged launches; the published "
                                                 "peak assumes 2.4 GHz"})
        # kernel-only duration and HBM traffic from committed rocprofv3 summaries, while the kernel is unchanged
        k_us = stored_profile("kernel_us", f"{family}_{tag}")
        roof["rocprof_avg_kernel_us"] = k_us
        roof["frac_rocprof"] = (roof["frac"] * dom_us / k_us) if k_us else None
        roof["traffic"] = stored_profile("hbm_bytes", f"{family}_{tag}")
        step = {"value": flop / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s", "ms_per_step": ms_per_step,
                "ms_per_step_events": ms_per_step_events,
                "flop_per_step": flop, "roofline": roof,
                "per_launch_us": us,
                "per_launch_roofline_frac": {c.name: c.flops / (us[c.name] * 1e-6) / 1e12 / c.roof_tf for c in cases},
                "launch": {c.name: c.plan.describe(c.which) for c in cases}}
        return step, cases

    steps = {}
    step_cases = {}
    for bf16 in (False, True):
        tag = "bf16" if bf16 else "f32"
        if args.dtype in (tag, "both"):
            steps[tag], step_cases[tag] = run_step(bf16)
    head_tag = "f32" if "f32" in steps else "bf16"
    head = steps[head_tag]

    out = {
        "metric": "operator fwd+bwd TFLOP/s (or GB/s) & % of roofline at ResNet-style layer shapes",
        "value": head["value"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head_tag, "data": "synthetic",
        "config": {"workload": "configs[1]: conv-equivalent Syno operator (Unfold 3x3 pad 1, Share, Reduce C,kh,kw), "
                               "forward + backward-data + backward-weight, N=32, ResNet-18 stages (64,56) (128,28) "
                               "(256,14) (512,7); " + ("fp32" if head_tag == "f32" else "bf16 inputs, fp32 accumulation")
                               + "; buffers rotate over %.0f MB per call" % args.rotate_mb,
                   "flop_per_step": head["flop_per_step"]},
        "roofline": head["roofline"],
        "per_launch_us": head["per_launch_us"],
        "per_launch_roofline_frac": head["per_launch_roofline_frac"],
    }
    if head_tag == "f32" and "bf16" in steps:
        out["bf16"] = steps["bf16"]        # the same step with bf16 inputs and fp32 accumulation, timed separately

    def event_us(fn, iters):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / iters * 1e3

    # ---- practical ceilings of this machine, measured in the same run ---------------------------------------------
    ceilings = {}
    for tag, dt in (("f32", F32), ("bf16", BF16)):
        flop, launch = syno.mfma_rate(dt, iters=2000, workgroups=512)
        ceilings[f"mfma_only_loop_{tag}_TFLOP/s"] = flop / (event_us(launch, 5) * 1e-6) / 1e12
    for mib in (24, 64, 256, 1024):
        srcs = [torch.empty(mib << 20, dtype=torch.uint8, device=dev).fill_(1) for _ in range(max(2, 1024 // mib // 2))]
        dsts = [torch.empty_like(s) for s in srcs]
        k = [0]

        def copy():
            dsts[k[0] % len(dsts)].copy_(srcs[k[0] % len(srcs)])
            k[0] += 1

        def fill():
            dsts[k[0] % len(dsts)].fill_(2)
            k[0] += 1

        ceilings[f"device_copy_{mib}MiB_GB/s"] = 2 * (mib << 20) / (event_us(copy, 30) * 1e-6) / 1e9     # read + write
        ceilings[f"device_fill_{mib}MiB_GB/s"] = (mib << 20) / (event_us(fill, 30) * 1e-6) / 1e9
        del srcs, dsts
    one = torch.zeros(1, device=dev)
    ceilings["smallest_launch_us"] = event_us(lambda: one.add_(1.0), 200)    # back-to-back one-element kernels
    out["ceilings"] = ceilings

    # ---- detail: every workload, per call -----------------------------------------------------------------
    if not args.no_detail:
        detail = []
        want = lambda i: args.config in (-1, i)
        cases = []
        if want(0):
            cases.append(Case("config0_conv16_f32_fwd", wl.config0(), 0))
        if want(1):
            for tag in steps:
                cases += step_cases[tag]
            for stage, (C, H) in enumerate(wl.RESNET18_STAGES):     # bf16 results as well (changes the byte count)
                w = wl.make_conv(32, C, H, seed=0, bf16=True, out_bf16=True)
                cases.append(Case(f"conv3x3_C{C}_{H}x{H}_N32_bf16_out_bf16_fwd", w, 0))
            # the downsampling convolutions between the first two stages (a Stride below the window): forward on the
            # contraction kernel, the gradients at stride 1 on the stride's phase planes
            for bf16 in (False, True):
                for K in (3, 1):
                    w = wl.make_conv(32, 64, 28, seed=0, bf16=bf16, Co=128, K=K, stride=2, with_grad=True)
                    cases += [Case(f"conv{K}x{K}_stride2_C64_Co128_56to28_N32_{'bf16' if bf16 else 'f32'}_{PASS[k]}", w, k)
                              for k in range(3)]
        if want(2):
            cases.append(Case("config2_gshift_bf16_N32_fwd", wl.config2(), 0))
            cases.append(Case("config2_gshift_bf16_N32_out_bf16_fwd", wl.make_gshift(32, seeds=(0, 0, 0), out_bf16=True), 0))
        if want(3):
            w3 = wl.config3_train()
            cases += [Case(f"config3_depthwise_s2_f32_{PASS[k]}", w3, k) for k in range(3)]
        if want(4):
            w4 = wl.config4()
            cases += [Case(f"config4_gshift_bf16_N128_{PASS[k]}", w4, k) for k in range(3)]
        if args.config == -1:
            # the matrix product the paper substitutes in GPT-2 (QKV projection, 8192 tokens), all three passes
            for bf16 in (False, True):
                wq = wl.qkv_projection(bf16)
                cases += [Case(f"qkv_mm_8192x768x2304_{'bf16' if bf16 else 'f32'}_{PASS[k]}", wq, k, sets=2)
                          for k in range(3)]
        for c in cases:
            med, _ = c.time_us(40)
            row = c.row(med)
            if c.bound == "hbm":      # the same call replayed on one buffer set: out of the last-level cache
                row["us_hot_cache"] = c.time_us(40, hot=True)[0]
            detail.append(row)
        if want(4):
            t = {r["case"]: r for r in detail}
            k4 = [f"config4_gshift_bf16_N128_{p}" for p in PASS]
            us4 = sum(t[k]["us"] for k in k4)
            detail.append({"case": "config4_gshift_bf16_N128_training_step (sum of the three calls)", "us": us4,
                           "TFLOP/s": 3 * wl.config4().flops / (us4 * 1e-6) / 1e12,
                           "GB/s": sum(t[k]["GB/s"] * t[k]["us"] for k in k4) / us4, "bound": "hbm",
                           "roofline_frac": sum(t[k]["GB/s"] * t[k]["us"] for k in k4) / us4 / HBM_PEAK_GBS})
        if args.config == -1:
            # Operator 1 (two stages, two weights) in place of the first stage's convolution: the forward sweep and
            # the backward sweep (dX and both weight gradients), each timed as a whole
            for bf16 in (False, True):
                w = wl.operator1(0, bf16)
                chain = syno.Chain(w.descs)
                eb = 2 if bf16 else 4
                X, G = to_dev(w.X, w.X_bits), to_dev(w.G, w.G_bits)
                Ws = [to_dev(v, b) for v, b in zip(w.Ws, w.Ws_bits or [None, None])]
                out0, acts0 = chain.forward(X, Ws)
                sets = [(X.clone(), [a.clone() for a in acts0], G.clone(), torch.empty_like(out0), torch.empty_like(X))
                        for _ in range(4)]
                n_x, n_z, n_o = (int(np.prod(t)) for t in (w.x_shape, w.inter_shapes[0], w.out_shape))
                n_w = sum(int(np.prod(t)) for t in w.w_shapes)
                sweeps = {
                    "fwd": (lambda t: chain.forward(t[0], Ws, acts=t[1], out=t[3]), w.flops,
                            eb * (n_x + 2 * n_z + n_o + n_w)),
                    # stage 2: read G, Z, W2, write dZ, dW2; stage 1: read dZ (twice), X, W1, write dX, dW1
                    "bwd": (lambda t: chain.backward(t[0], Ws, t[1], t[2], dX=t[4]), 2 * w.flops,
                            eb * (2 * n_o + 4 * n_z + 2 * n_x + n_w) + 4 * n_w),
                }
                for tag, (fn, flops, nbytes) in sweeps.items():
                    it = [0]

                    def sweep():
                        fn(sets[it[0] % 4])
                        it[0] += 1

                    us_s = event_us(sweep, 20)
                    which = (0,) if tag == "fwd" else (2, 1)
                    detail.append({"case": f"operator1_C64_56x56_N32_{'bf16' if bf16 else 'f32'}_{tag}_sweep",
                                   "kernel": " + ".join(p.kernel(k) for p in chain.stages for k in which),
                                   "launch": " | ".join(p.describe(k) for p in chain.stages for k in which),
                                   "us": us_s, "TFLOP/s": flops / (us_s * 1e-6) / 1e12,
                                   "GB/s": nbytes / (us_s * 1e-6) / 1e9, "bound": "hbm",
                                   "roofline_frac": nbytes / (us_s * 1e-6) / 1e9 / HBM_PEAK_GBS, "rotating_sets": 4})
            # pure views (no Reduce) on the view kernel: a cyclic shift with a per-channel scale and a
            # space-to-depth rearrangement, both 102.8 MB in and out
            for name, dv in (("shift_scale_C128_56x56_N64_f32", wl.shifted_scale(64, 128, 56, 56)),
                             ("pixel_unshuffle_C128_28x28_r2_N64_f32", wl.pixel_unshuffle(64, 128, 28, 28, 2))):
                pv = syno.Plan(dv)
                sets_v = [(torch.randn(pv.x_shape, device=dev), torch.randn(pv.w_shape if pv.w_shape else (1,), device=dev),
                           torch.empty(pv.out_shape, device=dev)) for _ in range(4)]
                nb = 4 * (int(np.prod(pv.x_shape)) + int(np.prod(pv.out_shape)))
                # forward reads X through the view and writes the result in runs; backward-data (both views are
                # one-to-one) reads the gradient in runs and scatters dX through the same tables
                # backward-weight reads the gradient and X and leaves one sum per weight element
                dws = [torch.empty(pv.w_shape if pv.w_shape else (1,), device=dev) for _ in range(4)]
                for which, tag in ((0, "_fwd"), (1, "_bwd_data"), (2, "_bwd_weight")):
                    calls = [pv.bind(0, a, b, o) if which == 0 else pv.bind(1, o, b, a) if which == 1 else pv.bind(2, a, o, dw)
                             for (a, b, o), dw in zip(sets_v, dws)]
                    it = [0]

                    def run_view():
                        calls[it[0] % 4]()
                        it[0] += 1

                    us_v = event_us(run_view, 12)
                    detail.append({"case": name + tag, "kernel": pv.kernel(which), "launch": pv.describe(which), "us": us_v,
                                   "GB/s": nb / (us_v * 1e-6) / 1e9, "bound": "hbm",
                                   "roofline_frac": nb / (us_v * 1e-6) / 1e9 / HBM_PEAK_GBS, "rotating_sets": 4})
            # the materialised-reduction pass on a convolution of 2x2 block sums (one loop nest with five Reduces):
            # the graph as written runs on the index-program kernel, the chain the library cuts it into on two small
            # reduction stages and the contraction kernel
            dpc = wl.pooled_conv2d(32, 64, 64, 28, 28, 2, 3)
            whole, mat = syno.Plan(dpc), syno.Chain.materialized(dpc)
            Xp = torch.randn(whole.x_shape, device=dev)
            Wp = torch.randn(whole.w_shape, device=dev) * 0.05
            Wsp = [Wp if i == mat.weight_stage else None for i in range(len(mat.stages))]
            o1 = whole.forward(Xp, Wp)
            o2, acts_p = mat.forward(Xp, Wsp)
            torch.cuda.synchronize()
            agree = float((o1 - o2).norm() / o1.norm())
            us_whole = event_us(lambda: whole.forward(Xp, Wp, out=o1), 3)
            us_chain = event_us(lambda: mat.forward(Xp, Wsp, acts=acts_p, out=o2), 20)
            fl_whole = 2 * int(np.prod(whole.out_shape)) * 64 * 9 * 4
            detail.append({"case": "pooled_conv_C64_28x28_N32_f32_fwd: single loop nest vs materialised chain",
                           "kernel": whole.kernel(0) + " vs " + " + ".join(p.kernel(0) for p in mat.stages),
                           "us_single_loop_nest": us_whole, "us": us_chain, "stages": len(mat.stages),
                           "TFLOP/s": fl_whole / (us_chain * 1e-6) / 1e12, "rel_l2_between_the_two": agree,
                           "note": "TFLOP/s counts the multiply-adds of the single loop nest"})
        out["detail"] = detail

    # ---- CPU baseline: the checker as it stands, on a bounded sample of the same workload ---------------------
    if not args.no_cpu_baseline:
        import oracle
        n_s = 1 << 18
        rng = np.random.default_rng(0)
        macs, t_cpu = 0, 0.0
        for stage in range(4):
            w = wl.config1_train(stage, False)
            n_o, k_red = int(np.prod(w.out_shape)), w.flops // 2 // int(np.prod(w.out_shape))
            idx = rng.integers(0, n_o, n_s)
            xs = np.unique(rng.integers(0, int(np.prod(w.x_shape)), 4096))
            ws = np.unique(rng.integers(0, int(np.prod(w.w_shape)), 4096))
            Xd, Wd, Gd = w.X.astype(np.float64), w.W.astype(np.float64), w.G.astype(np.float64)
            t = time.perf_counter()
            oracle.forward_at(w.desc, Xd, Wd, idx)
            if stage >= 2:      # the scatter-form gradients walk the whole loop nest whatever is sampled
                oracle.backward(w.desc, Xd, Wd, Gd, x_sample=xs, w_sample=ws)
            t_cpu += time.perf_counter() - t
            macs += n_s * k_red + (n_o * k_red if stage >= 2 else 0)
        out["cpu_baseline"] = {"value": 2 * macs / t_cpu / 1e12, "unit": "TFLOP/s", "cores": oracle.threads(),
                               "kind": "oracle", "seconds": t_cpu,
                               "sample": f"forward at {n_s} sampled outputs of each of the four configs[1] shapes, and the whole "
                                         f"backward loop nest (both gradients accumulated at 4096 sampled elements each) of the "
                                         f"14x14 and 7x7 shapes; fp64 loop-nest interpreter; {macs} loop-nest points, "
                                         f"counted as one multiply-add each"}
        if not args.no_detail and args.config == -1:
            per_config = {}
            for name, w, full in (("config0", wl.config0(), True), ("config2", wl.config2(), False),
                                  ("config3", wl.config3(), False), ("config4", wl.config4(), False)):
                n_o = int(np.prod(w.out_shape))
                idx = np.arange(n_o) if full else rng.integers(0, n_o, n_s)
                t = time.perf_counter()
                oracle.forward_at(w.desc, w.X.astype(np.float64), w.W.astype(np.float64), idx)
                dt = time.perf_counter() - t
                per_config[name] = {"forward_outputs": int(idx.size), "seconds": dt,
                                    "GFLOP/s": 2 * idx.size * (w.flops // 2 // n_o) / dt / 1e9}
            out["cpu_baseline"]["per_config_forward"] = per_config
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
