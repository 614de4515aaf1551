#!/usr/bin/env python3
"""Benchmark: operator evaluation throughput on one MI355X.

A step is one evaluation of the conv-equivalent synthesized operator (Unfold 3x3, Share, Reduce over
C,kh,kw) at the four ResNet-18 stage shapes with N=32, each once in fp32 and once with bf16 inputs and
fp32 accumulation.  Inputs are synthetic, seeded, and resident in HBM before the timed region.  The other
workloads (grouped shift-unfold forward and training step, strided depthwise) are timed separately and
reported under "detail".  Prints one JSON line.
"""
from __future__ import annotations

import argparse
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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
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
    from syno_inputs import BF16, workloads as wl
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from util import to_dev

    if not os.path.exists(syno.library_path()):
        from paper_2410_23745_amd import build
        build.build()
    syno.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    class Case:
        """One operator call with its device buffers (several rotating sets so that memory-bound calls do not
        replay out of the 256 MB last-level cache)."""

        def __init__(self, name, w, which, sets=1):
            self.name, self.w, self.which = name, w, which
            self.plan = syno.Plan(w.desc)
            inb = 2 if w.desc.in_dtype == BF16 else 4
            outb = 2 if (w.desc.out_dtype == BF16 and which != 2) else 4
            self.bytes = alg_bytes(w, which, inb, outb)
            self.flops = w.flops
            self.dtype = "bf16" if w.desc.in_dtype == BF16 else "f32"
            X, W = to_dev(w.X, w.X_bits), to_dev(w.W, w.W_bits)
            G = to_dev(w.G, w.G_bits) if w.G is not None else None
            self.sets = []
            for _ in range(sets):
                a, b = ((X, W), (G, W), (X, G))[which]
                out_shape = (w.out_shape, w.x_shape, w.w_shape)[which]
                out_dtype = torch.float32 if which == 2 else self.plan.out_dtype
                self.sets.append((a.clone(), b.clone(), torch.empty(out_shape, dtype=out_dtype, device=dev)))
            self.fn = (self.plan.forward, self.plan.backward_data, self.plan.backward_weight)[which]
            self.kernel = self.plan.kernel(which)
            self.i = 0

        def launch(self):
            a, b, o = self.sets[self.i % len(self.sets)]
            self.i += 1
            self.fn(a, b, o)

        def time_ms(self, iters, warm=3):
            for _ in range(warm):
                self.launch()
            torch.cuda.synchronize()
            marks = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
            marks[0].record()
            for i in range(iters):
                self.launch()
                marks[i + 1].record()
            torch.cuda.synchronize()
            evs = list(zip(marks[:-1], marks[1:]))
            t = sorted(s.elapsed_time(e) for s, e in evs)
            return t[len(t) // 2], sum(t) / len(t)

    # ---- the timed step: configs[1] --------------------------------------------------------------------
    step_cases = []
    for bf16 in (False, True):
        for stage, (C, H) in enumerate(wl.RESNET18_STAGES):
            step_cases.append(Case(f"conv3x3_C{C}_{H}x{H}_N32_{'bf16' if bf16 else 'f32'}", wl.config1(stage, bf16), 0))
    step_flops = sum(c.flops for c in step_cases)

    def one_step():
        for c in step_cases:
            c.launch()

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    ev = {c.name: [] for c in step_cases}
    t0 = time.perf_counter()
    for _ in range(args.steps):
        # one event between consecutive launches (on the current stream, which is the stream the binding launches
        # on): launch i is bracketed by events i and i+1
        prev = torch.cuda.Event(enable_timing=True)
        prev.record()
        for c in step_cases:
            c.launch()
            e = torch.cuda.Event(enable_timing=True)
            e.record()
            ev[c.name].append((prev, e))
            prev = e
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = step_flops / (ms_per_step * 1e-3) / 1e12

    per_case = {}
    for c in step_cases:
        ts = [s.elapsed_time(e) for s, e in ev[c.name]]
        per_case[c.name] = sum(ts) / len(ts)
    # dominant kernel of the step = the family with the largest summed duration
    fam_time = {}
    for c in step_cases:
        fam_time.setdefault((c.kernel, c.dtype), []).append(c)
    dom_key = max(fam_time, key=lambda k: sum(per_case[c.name] for c in fam_time[k]))
    dom = fam_time[dom_key]
    dom_ms = sum(per_case[c.name] for c in dom) / len(dom)
    dom_flops = sum(c.flops for c in dom) / len(dom)
    dom_bytes = sum(c.bytes for c in dom) / len(dom)
    mfma_peak = MFMA_PEAK_TFLOPS[dom_key[1]]
    # which roof binds the dominant kernel: min(peak, AI * BW)
    ai = dom_flops / dom_bytes
    if ai * HBM_PEAK_GBS / 1e3 < mfma_peak:
        ach = dom_bytes / (dom_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                    "traffic": None}
    else:
        ach = dom_flops / (dom_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": ach, "peak": mfma_peak, "unit": "TFLOP/s", "frac": ach / mfma_peak,
                    "traffic": None}
    roofline["kernel"] = f"{dom_key[0]}[{dom_key[1]}]"
    roofline["avg_launch_us"] = dom_ms * 1e3
    roofline["launches_averaged"] = [c.name for c in dom]
    # HBM traffic per launch comes from stored rocprofv3 --pmc runs (the record at the end of
    # profiles/hbm_traffic_all_workloads.txt) and only counts while the kernel sources it was taken on are unchanged
    try:
        import hashlib
        rec = {}
        for line in open(os.path.join(ROOT, "profiles", "hbm_traffic_all_workloads.txt")):
            key, sep, val = line.partition(":")
            if sep and key in ("kernel", "hbm_bytes_per_launch", "sources", "sha256"):
                rec[key] = val.split("(")[0].strip() if key == "hbm_bytes_per_launch" else val.strip()
        srcs = [os.path.join(ROOT, "paper_2410_23745_amd", "csrc", f) for f in rec["sources"].split()]
        digest = hashlib.sha256(b"".join(open(f, "rb").read() for f in srcs)).hexdigest()
        if digest == rec["sha256"] and rec["kernel"] == roofline["kernel"]:
            roofline["traffic"] = float(rec["hbm_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        pass

    out = {
        "metric": "operator fwd+bwd TFLOP/s (or GB/s) & % of roofline at ResNet-style layer shapes",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 and bf16-in/f32-acc", "data": "synthetic",
        "config": {"workload": "configs[1]: conv-equivalent Syno operator (Unfold 3x3 pad 1, Share, Reduce C,kh,kw), "
                               "forward (the passes this configuration names; the backward passes of the same shapes are timed "
                               "under detail), N=32, ResNet-18 stages (64,56) (128,28) (256,14) (512,7), fp32 and bf16 inputs",
                   "flop_per_step": step_flops},
        "roofline": roofline,
        "per_launch_us": {k: v * 1e3 for k, v in per_case.items()},
    }

    # ---- detail: every workload, per call -----------------------------------------------------------------
    if not args.no_detail:
        detail = []
        w2, w3, w4 = wl.config2(), wl.config3_train(), wl.config4()
        cases = [Case("config0_conv16_f32_fwd", wl.config0(), 0)] + step_cases + [
            Case("config2_gshift_bf16_N32_fwd", w2, 0, sets=8),
            Case("config3_depthwise_s2_f32_fwd", w3, 0, sets=6),
            Case("config4_gshift_bf16_N128_fwd", w4, 0, sets=8),
            Case("config4_gshift_bf16_N128_bwd_data", w4, 1, sets=8),
            Case("config4_gshift_bf16_N128_bwd_weight", w4, 2, sets=8),
            # backward passes of the first two shapes (not named by the configs; the metric is forward + backward)
            Case("config3_depthwise_s2_f32_bwd_data", w3, 1, sets=6),
            Case("config3_depthwise_s2_f32_bwd_weight", w3, 2, sets=6),
        ]
        for bf16 in (False, True):
            for stage, (C, H) in enumerate(wl.RESNET18_STAGES):
                wt = wl.config1_train(stage, bf16)
                tag = f"conv3x3_C{C}_{H}x{H}_N32_{'bf16' if bf16 else 'f32'}"
                cases.append(Case(tag + "_bwd_data", wt, 1))
                cases.append(Case(tag + "_bwd_weight", wt, 2))
        # the matrix product the paper substitutes in GPT-2 (QKV projection, 8192 tokens), all three passes
        for bf16 in (False, True):
            wq = wl.qkv_projection(bf16)
            for which, tag in enumerate(("fwd", "bwd_data", "bwd_weight")):
                cases.append(Case(f"qkv_mm_8192x768x2304_{'bf16' if bf16 else 'f32'}_{tag}", wq, which, sets=2))
        for c in cases:
            med, avg = c.time_ms(200, warm=10)
            tf = c.flops / (med * 1e-3) / 1e12
            gbs = c.bytes / (med * 1e-3) / 1e9
            peak = MFMA_PEAK_TFLOPS[c.dtype]
            roof_tf = min(peak, c.flops / c.bytes * HBM_PEAK_GBS / 1e3)
            detail.append({"case": c.name, "kernel": c.kernel, "launch": c.plan.describe(c.which), "us": med * 1e3,
                           "TFLOP/s": tf, "GB/s": gbs,
                           "bound": "hbm" if roof_tf < peak else "mfma", "roofline_frac": tf / roof_tf,
                           "rotating_sets": len(c.sets)})
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
                for i in range(3):
                    fn(sets[i % 4])
                torch.cuda.synchronize()
                marks = [torch.cuda.Event(enable_timing=True) for _ in range(21)]
                marks[0].record()
                for i in range(20):
                    fn(sets[i % 4])
                    marks[i + 1].record()
                torch.cuda.synchronize()
                ts = sorted(a.elapsed_time(b) for a, b in zip(marks[:-1], marks[1:]))
                med = ts[len(ts) // 2]
                which = (0,) if tag == "fwd" else (2, 1)
                detail.append({"case": f"operator1_C64_56x56_N32_{'bf16' if bf16 else 'f32'}_{tag}_sweep",
                               "kernel": " + ".join(p.kernel(k) for p in chain.stages for k in which),
                               "launch": " | ".join(p.describe(k) for p in chain.stages for k in which),
                               "us": med * 1e3, "TFLOP/s": flops / (med * 1e-3) / 1e12,
                               "GB/s": nbytes / (med * 1e-3) / 1e9, "rotating_sets": 4})
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
            for which, tag in ((0, "_fwd"), (1, "_bwd_data")):
                it = [0]

                def run_view():
                    a, b, o = sets_v[it[0] % 4]
                    it[0] += 1
                    if which == 0:
                        pv.forward(a, b, out=o)
                    else:
                        pv.backward_data(o, b, dX=a)

                run_view()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(12):
                    run_view()
                e1.record()
                torch.cuda.synchronize()
                us_v = e0.elapsed_time(e1) / 12 * 1e3
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

        def timed(fn, iters):
            fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(iters):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / iters * 1e3

        us_whole = timed(lambda: whole.forward(Xp, Wp, out=o1), 3)
        us_chain = timed(lambda: mat.forward(Xp, Wsp, acts=acts_p, out=o2), 20)
        fl_whole = 2 * int(np.prod(whole.out_shape)) * 64 * 9 * 4
        detail.append({"case": "pooled_conv_C64_28x28_N32_f32_fwd: single loop nest vs materialised chain",
                       "kernel": whole.kernel(0) + " vs " + " + ".join(p.kernel(0) for p in mat.stages),
                       "us_single_loop_nest": us_whole, "us": us_chain, "stages": len(mat.stages),
                       "TFLOP/s": fl_whole / (us_chain * 1e-6) / 1e12, "rel_l2_between_the_two": agree,
                       "note": "TFLOP/s counts the multiply-adds of the single loop nest"})
        out["detail"] = detail

    # ---- practical ceilings of this machine, measured in the same run with library-free torch ops ---------------
    if not args.no_detail:
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

        ceilings = {}
        for mib in (64, 256, 1024):
            src = torch.empty(mib << 20, dtype=torch.uint8, device=dev).fill_(1)
            dsts = [torch.empty_like(src) for _ in range(2)]
            k = [0]

            def copy():
                dsts[k[0] & 1].copy_(src)
                k[0] += 1

            us = event_us(copy, 20)
            ceilings[f"device_copy_{mib}MiB_GB/s"] = 2 * (mib << 20) / (us * 1e-6) / 1e9     # read + write
            del src, dsts
        one = torch.zeros(1, device=dev)
        ceilings["smallest_launch_us"] = event_us(lambda: one.add_(1.0), 200)    # back-to-back one-element kernels
        out["ceilings"] = ceilings

    # ---- CPU baseline: the checker as it stands, on a bounded sample of the same workload ---------------------
    if not args.no_cpu_baseline:
        import oracle
        n_s = 1 << 20
        rng = np.random.default_rng(0)
        macs, t_cpu = 0, 0.0
        for stage in range(4):
            w = wl.config1(stage, False)
            idx = rng.integers(0, int(np.prod(w.out_shape)), n_s)
            Xd, Wd = w.X.astype(np.float64), w.W.astype(np.float64)
            t = time.perf_counter()
            oracle.forward_at(w.desc, Xd, Wd, idx)
            t_cpu += time.perf_counter() - t
            macs += n_s * (w.flops // 2 // int(np.prod(w.out_shape)))
        out["cpu_baseline"] = {"value": 2 * macs / t_cpu / 1e12, "unit": "TFLOP/s", "cores": oracle.threads(),
                               "kind": "oracle", "seconds": t_cpu,
                               "sample": f"{n_s} sampled outputs of each of the four configs[1] shapes (fp64 loop-nest "
                                         f"interpreter; {macs} multiply-adds in total)"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
