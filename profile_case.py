"""Run one workload a few times so that rocprofv3 can attribute kernel time and HBM counters to it.

    rocprofv3 --kernel-trace --stats -- python3 profile_case.py config1_s0_f32 --iters 20
    rocprofv3 --pmc FETCH_SIZE       -- python3 profile_case.py config1_s0_f32 --iters 5 --copy
    rocprofv3 --pmc WRITE_SIZE       -- python3 profile_case.py config1_s0_f32 --iters 5 --copy

With --copy a plain device copy of a known size (256 MiB, `Tensor.copy_`) runs first; what FETCH_SIZE and
WRITE_SIZE report for it gives the factor that turns the counters into bytes.

Cases: config0, config1_s{0..3}_{f32|bf16}, config2, config3, config4_{fwd|bwd_data|bwd_weight}, and the backward
passes of the first two shapes with a seeded output gradient: config1t_s{0..3}_{f32|bf16}_{fwd|bwd_data|bwd_weight},
config3t_{fwd|bwd_data|bwd_weight}; Operator 1 (two stages) on a ResNet-18 stage shape: op1_s{0..3}_{f32|bf16}_{fwd|bwd}; the GPT-2 QKV projection as a matrix product:
qkv_{f32|bf16}_{fwd|bwd_data|bwd_weight}; the two pure views of the benchmark (102.8 MB in and out, random values):
view_{shift|unshuffle}_{fwd|bwd_data}; the library's MFMA-only loop (nothing but matrix instructions on every
SIMD: the reading that "always busy" gives for the matrix-unit counters): mfma_rate_{f32|bf16}.
Buffers rotate over several copies so that every launch reads HBM rather than the last-level cache.
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def make_case(name: str):
    from syno_inputs import workloads as wl
    which = 0
    if name == "config0":
        w = wl.config0()
    elif name.startswith("config1_s"):
        w = wl.config1(int(name[9]), name.endswith("bf16"))
    elif name.startswith("config1t_s"):     # config1t_s<stage>_<f32|bf16>_<fwd|bwd_data|bwd_weight>
        stage, dt, direction = int(name[10]), name[12:].split("_")[0], name[12:].split("_", 1)[1]
        w = wl.config1_train(stage, dt == "bf16")
        which = {"fwd": 0, "bwd_data": 1, "bwd_weight": 2}[direction]
    elif name.startswith("config3t_"):
        w = wl.config3_train()
        which = {"fwd": 0, "bwd_data": 1, "bwd_weight": 2}[name[9:]]
    elif name == "config2":
        w = wl.config2()
    elif name == "config3":
        w = wl.config3()
    elif name.startswith("qkv_"):            # qkv_<f32|bf16>_<fwd|bwd_data|bwd_weight>
        dt, direction = name[4:].split("_", 1)
        w = wl.qkv_projection(dt == "bf16")
        which = {"fwd": 0, "bwd_data": 1, "bwd_weight": 2}[direction]
    elif name.startswith("config4_"):
        w = wl.config4()
        which = {"fwd": 0, "bwd_data": 1, "bwd_weight": 2}[name[8:]]
    else:
        raise SystemExit(f"unknown case {name}")
    return w, which


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("case")
    ap.add_argument("--iters", type=int, default=10)
    ap.add_argument("--sets", type=int, default=6)
    ap.add_argument("--copy", action="store_true")
    args = ap.parse_args()
    import numpy as np
    import torch
    import paper_2410_23745_amd as syno
    from syno_inputs import BF16

    syno.load_library()
    dev = torch.device("cuda:0")
    if args.copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    def dev_t(vals, bits):
        if bits is not None:
            return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)
        return torch.from_numpy(np.ascontiguousarray(vals, dtype=np.float32)).to(dev)

    if args.case.startswith("mfma_rate_"):
        from syno_inputs import F32
        flop, launch = syno.mfma_rate(BF16 if args.case.endswith("bf16") else F32, iters=2000, workgroups=1024)
        for _ in range(args.iters):
            launch()
        torch.cuda.synchronize()
        print(f"{args.case}: {flop} flop per launch; {args.iters + 1} launches")
        return 0

    if args.case.startswith("op1_s"):       # op1_s<stage>_<f32|bf16>_<fwd|bwd>
        from syno_inputs import workloads as wl
        stage, dt, direction = int(args.case[5]), args.case[7:].split("_")[0], args.case[7:].split("_")[1]
        w = wl.operator1(stage, dt == "bf16")
        chain = syno.Chain(w.descs)
        X, G = dev_t(w.X, w.X_bits), dev_t(w.G, w.G_bits)
        Ws = [dev_t(v, b) for v, b in zip(w.Ws, w.Ws_bits or [None, None])]
        out, acts = chain.forward(X, Ws)
        sets = [(X.clone(), [a.clone() for a in acts], G.clone(), torch.empty_like(out), torch.empty_like(X))
                for _ in range(args.sets)]
        for i in range(args.iters):
            s = sets[i % len(sets)]
            if direction == "fwd":
                chain.forward(s[0], Ws, acts=s[1], out=s[3])
            else:
                chain.backward(s[0], Ws, s[1], s[2], dX=s[4])
        torch.cuda.synchronize()
        print(f"{args.case}: " + " | ".join(p.describe(k) for p in chain.stages
                                            for k in ((0,) if direction == "fwd" else (2, 1))))
        return 0

    if args.case.startswith("view_"):       # view_<shift|unshuffle>_<fwd|bwd_data>
        from syno_inputs import workloads as wl
        kind, direction = args.case[5:].split("_", 1)
        d = wl.shifted_scale(64, 128, 56, 56) if kind == "shift" else wl.pixel_unshuffle(64, 128, 28, 28, 2)
        which = {"fwd": 0, "bwd_data": 1}[direction]
        plan = syno.Plan(d)
        fn = (plan.forward, plan.backward_data)[which]
        shapes = ((plan.x_shape, plan.out_shape), (plan.out_shape, plan.x_shape))[which]
        sets = [(torch.randn(shapes[0], device=dev), torch.randn(plan.w_shape if plan.w_shape else (1,), device=dev),
                 torch.empty(shapes[1], device=dev)) for _ in range(args.sets)]
        for i in range(args.iters):
            s = sets[i % len(sets)]
            fn(s[0], s[1], s[2])
        torch.cuda.synchronize()
        print(f"{args.case}: {plan.describe(which)}; {args.iters} launches")
        return 0

    w, which = make_case(args.case)

    plan = syno.Plan(w.desc)
    X, W = dev_t(w.X, w.X_bits), dev_t(w.W, w.W_bits)
    G = dev_t(w.G, w.G_bits) if w.G is not None else None
    a, b = ((X, W), (G, W), (X, G))[which]
    fn = (plan.forward, plan.backward_data, plan.backward_weight)[which]
    out_shape = (w.out_shape, w.x_shape, w.w_shape)[which]
    out_dtype = torch.float32 if which == 2 else plan.out_dtype
    sets = [(a.clone(), b.clone(), torch.empty(out_shape, dtype=out_dtype, device=dev)) for _ in range(args.sets)]
    for i in range(args.iters):
        s = sets[i % len(sets)]
        fn(s[0], s[1], s[2])
    torch.cuda.synchronize()
    print(f"{args.case}: {plan.describe(which)}; {args.iters} launches")
    return 0


if __name__ == "__main__":
    sys.exit(main())
