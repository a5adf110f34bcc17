#!/usr/bin/env python3
"""Benchmark of the conv3d hot path on one MI355X.

Workload (default): the CosmoFlow-shaped network step — N=4 samples of 4x128^3, five
conv3d 3x3x3 + leaky-ReLU + 2x2x2 avg-pool stages (16..256 channels), dense 16384-2048-256-4,
MSE; bf16 storage, fp32 accumulation; forward + backward (BD and BF of every layer).
A step = one pass of that whole path over one synthetic batch already resident in HBM.

Prints ONE JSON line: conv3d fwd+bwd TFLOP/s of the step (conv flops by Table I's convention,
2*27*Cin*Cout per output voxel and pass, divided by the whole step time), voxels/s, a per-call
table, the roofline of the dominant call (timed with HIP events inside the timed region) and
the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_BF16_TFLOPS = 2500.0
PEAK_FP32_VALU_TFLOPS = 157.3
RIDGE = PEAK_MFMA_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)


def cpu_baseline(seed):
    """The oracle, as it stands, on a bounded sample: stage 2 of the stack (16->32 channels on 64^3),
    the whole batch of four samples, all three passes (FP, BD, BF): about 10 s on the GPU machine's host cores."""
    import numpy as np
    import oracle as orc
    import synth
    from synth import recipes
    w, b = recipes.conv_params(seed, 102, 16, 32)
    w = synth.round_bf16(w).astype(np.float64)
    x = orc.Slab(synth.round_bf16(synth.slab("cosmo", seed, 7, (4, 16, 64, 64, 64), 0, 64)).astype(np.float64))
    dz = orc.Slab(synth.round_bf16(synth.slab("normal", seed, 8, (4, 32, 64, 64, 64), 0, 64)).astype(np.float64))
    t0 = time.time()
    z = orc.conv3d_fwd(x, w, b, act=orc.ACT_LEAKY, alpha=0.01)
    orc.conv3d_bwd_data(dz, z, w, act=orc.ACT_LEAKY, alpha=0.01)
    orc.conv3d_bwd_filter(x, dz, z, act=orc.ACT_LEAKY, alpha=0.01)
    dt = time.time() - t0
    flops = 3 * orc.conv_flops(16, 32, 4 * 64 ** 3)
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": "stage-2 conv (16->32 ch, 64^3, 4 samples) fwd+bwd_data+bwd_filter, fp64 direct loops",
            "seconds": round(dt, 2), "voxels_per_s": 4 * 64 ** 3 / dt}


def side_workload(args, seed):
    """Per-call tables for the other configurations (not the headline line)."""
    import numpy as np
    import torch
    import synth
    from synth import recipes
    import paper_2007_12856_amd as h3d
    from paper_2007_12856_amd.nets import SingleLayer, UNetLevel
    bf = torch.bfloat16
    if args.workload == "shard512":
        net = SingleLayer(1, 4, 16, 64, 512, 64, 512, seed=seed, faces_hw=True)
        name = "one 8-way depth shard of a 4x512^3 sample: 4x66x512x512 bf16, conv 4->16 + leaky + avg-pool, D halo faces; H and W faces of g"
    elif args.workload == "split256":
        net = SingleLayer(1, 64, 64, 32, 256, 32, 256, pool=False, seed=seed, split=True)
        name = "one 8-way depth shard of a 64-channel 256^3 sample: conv 64->64 whole, and as main planes + two 1-plane strips"
    elif args.workload == "bn":
        from paper_2007_12856_amd.nets import BatchNormLayer
        net = BatchNormLayer(4, 16, 128, 128, seed=seed)
        name = "local batch-normalisation passes on the first convolution's output: 4 x 16 x 128^3 bf16"
    elif args.workload == "table1":
        # the seven convolutions of Table I (fourth one with a stride of 2, no convolution biases, pooling until the
        # volume is 2^3), dense head 2048-256-4, on whole samples of --width^3 (128 or 256)
        from paper_2007_12856_amd.nets import CosmoFlowStack
        dev = lambda a, dt=bf: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(dt)
        channels, strides, pools, flat_w = recipes.table1_layout(args.width)
        P = recipes.cosmoflow_params(seed, args.width, channels, recipes.COSMO_FC, flat_w)
        x, t = recipes.cosmoflow_batch(seed, args.batch, args.width)
        net = CosmoFlowStack(dev(x), dev(t, torch.float32), [(dev(w), None) for w, _ in P["conv"]],
                             [(dev(w), dev(b, torch.float32)) for w, b in P["fc"]], fuse_pool=not args.unfused,
                             strides=strides, pools=pools)
        name = (f"network of Table I for {args.width}^3 inputs, N={args.batch}: conv 16-32-64-128(stride 2)-256-256-256, no conv biases, "
                f"leaky-ReLU, avg-pool, dense 2048-256-4, MSE; fwd+bwd; {net.conv_flops() / args.batch / 1e9:.2f} conv GFlop per sample")
    elif args.workload == "chain512":
        # the spatially-partitioned front of Table I's 512^3 network on one interior shard of an 8-way depth partition
        from paper_2007_12856_amd.nets import CosmoFlowShardChain
        dev = lambda a, dt=bf: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(dt)
        x, conv, dout, faces = recipes.shard_chain_inputs(seed, 512, 64, 64, 512, n=args.batch)
        net = CosmoFlowShardChain(h3d.Slab(dev(x), 1, 1, 64, 512), [(dev(w), None) for w, _ in conv], dev(dout),
                                  {k: (dev(lo), dev(hi)) for k, (lo, hi) in faces.items()}, fuse_pool=not args.unfused)
        name = (f"conv1-pool1 .. conv3-pool3 of Table I's 512^3 network on one interior shard of an 8-way depth partition "
                f"(N={args.batch} x 4x(64+2)x512x512 bf16), halo faces packed and unpacked per stage, fwd+bwd")
    elif args.workload == "xent":
        # segmentation loss on the output shard of the U-Net shape: 3 classes, 64 x 256 x 256 voxels of a 256^3 volume
        class _Xent:
            def __init__(self):
                g = torch.Generator(device="cuda")
                g.manual_seed(seed)
                z = h3d.Slab((3.0 * torch.randn((1, 3, 64, 256, 256), generator=g, device="cuda")).to(bf), 0, 0, 64, 256)
                lab = torch.randint(0, 3, (1, 64, 256, 256), generator=g, device="cuda", dtype=torch.uint8)
                dz, loss, ws = h3d.Slab(torch.empty_like(z.t), 0, 0, 64, 256), torch.zeros(1, device="cuda"), h3d.Workspace()
                nb = 2 * z.t.numel() * 2 + lab.numel()
                self.keep = (z, lab, dz, loss)
                self.ops = [{"name": "softmax_xent_fwd_bwd", "fn": lambda: h3d.softmax_xent_fwd_bwd(z, lab, 256 ** 3, loss, dz, ws),
                             "flops": 0, "bytes": nb}]

            def step(self):
                self.ops[0]["fn"]()

            def conv_flops(self):
                return 0
        net = _Xent()
        name = "softmax cross-entropy, forward + gradient, 3 classes on a 64x256x256 shard of a 256^3 volume, bf16"
    elif args.workload == "k5":
        # 5x5x5 filters (two halo planes): conv 32 -> 32 on a 32-plane interior shard of a 128^3 volume, the three passes
        class _K5:
            def __init__(self):
                g = torch.Generator(device="cuda")
                g.manual_seed(seed)
                rnd = lambda *sh: torch.randn(sh, generator=g, device="cuda")
                ci = co = 32
                geo = (2, 2, 32, 128)
                x = h3d.Slab(rnd(1, ci, 36, 128, 128).to(bf), *geo)
                z = h3d.Slab(rnd(1, co, 36, 128, 128).to(bf), *geo)
                dz = h3d.Slab(rnd(1, co, 36, 128, 128).to(bf), *geo)
                dx = h3d.Slab(torch.empty_like(x.t), *geo)
                zo = h3d.Slab(torch.empty_like(z.t), *geo)
                w = (rnd(co, ci, 5, 5, 5) * (2.0 / (125 * ci)) ** 0.5).to(bf)
                b = torch.zeros(co, device="cuda")
                dw, db = torch.empty((co, ci, 5, 5, 5), device="cuda"), torch.empty(co, device="cuda")
                ws = h3d.Workspace()
                fl = 2 * 125 * ci * co * 32 * 128 * 128
                nb = 2 * 36 * 128 * 128 * 2 * ci
                self.keep = (x, z, dz, dx, zo, w, b, dw, db)
                self.ops = [
                    {"name": "k5_fwd", "fn": lambda: h3d.conv3d_k5_fwd(x, w, b, zo, h3d.ACT_LEAKY, 0.01, ws), "flops": fl, "bytes": nb},
                    {"name": "k5_bwd_data", "fn": lambda: h3d.conv3d_k5_bwd_data(dz, z, w, dx, h3d.ACT_LEAKY, 0.01, ws), "flops": fl, "bytes": nb * 3 // 2},
                    {"name": "k5_bwd_filter", "fn": lambda: h3d.conv3d_k5_bwd_filter(x, dz, z, dw, db, h3d.ACT_LEAKY, 0.01, ws), "flops": fl, "bytes": nb * 3 // 2},
                ]

            def step(self):
                for o in self.ops:
                    o["fn"]()

            def conv_flops(self):
                return sum(o["flops"] for o in self.ops)
        net = _K5()
        name = "5x5x5 convolution 32->32, 32-plane interior shard (+2 halo planes per side) of a 128^3 volume, bf16, three passes"
    elif args.workload == "late256":
        net = SingleLayer(8, 256, 256, 16, 16, 0, 16, pool=False, seed=seed)
        name = "late layer N=8, 256->256, 16^3 bf16"
    else:
        dev = lambda a, dt=bf: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(dt)
        x, P, dout, faces = recipes.unet_level_inputs(seed, 256, 64, 64, 256)
        net = UNetLevel(h3d.Slab(dev(x), 2, 2, 64, 256), {k: (dev(w), dev(b, torch.float32)) for k, (w, b) in P.items()},
                        dev(dout), {k: tuple(None if f is None else dev(f) for f in pr) for k, pr in faces.items()})
        name = "U-Net-shaped level on a 64x256x256 shard of a 256^3 volume (halo 2), bf16, fwd+bwd"
    stream = torch.cuda.current_stream()
    if hasattr(net, "overlap") and not args.only:
        # the stack's second stream (late backward-filter calls, dense weight gradients): their table rows then show the
        # launch only, the "join" row the wait for them
        net.overlap = not args.no_overlap
    for _ in range(args.warmup):
        net.step()
    torch.cuda.synchronize()
    if args.only:
        sel = [o for o in net.ops if o["name"] == args.only]
        if not sel:
            sys.exit(f"bench.py: --only must be one of {[o['name'] for o in net.ops]}")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(args.steps):
            sel[0]["fn"]()
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        print(json.dumps({"metric": "single call", "kernel": args.only, "ms": ms, "steps": args.steps,
                          "tflops": sel[0]["flops"] / ms / 1e9, "config": {"workload": name}}))
        return
    tot = {o["name"]: 0.0 for o in net.ops}
    t0 = time.perf_counter()
    for _ in range(args.steps):
        evs = []
        for o in net.ops:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            o["fn"]()
            e1.record(stream)
            evs.append((o, e0, e1))
        torch.cuda.synchronize()
        for o, e0, e1 in evs:
            tot[o["name"]] += e0.elapsed_time(e1)
    dt = time.perf_counter() - t0
    per_call = []
    for o in net.ops:
        ms = tot[o["name"]] / args.steps
        per_call.append({"name": o["name"], "ms": round(ms, 4), "tflops": round(o["flops"] / ms / 1e9, 1) if o["flops"] else None,
                         "gbs": round(o["bytes"] / ms / 1e6, 1) if o["bytes"] else None})
    ms_step = sum(tot.values()) / args.steps
    print(json.dumps({"metric": "conv3d fwd+bwd TFLOP/s", "value": net.conv_flops() / ms_step / 1e9, "unit": "TFLOP/s", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": name}, "per_call": per_call}))


def measured_traffic(workload, call):
    """HBM bytes per launch of `call`, as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and scaled by the
    plain-copy factors; read from the 'TRAFFIC <call> <bytes>' lines of profiles/<workload>_step_hbm_traffic.txt.
    None when no measurement of that call is on record."""
    path = os.path.join(ROOT, "profiles", f"{workload}_step_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) == 3 and f[0] == "TRAFFIC" and f[1] == call:
            return int(f[2])
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=4)
    ap.add_argument("--width", type=int, default=128)
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "f32"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", default=None, help="after warm-up, time only this call of the step (name as in per_call); "
                    "used to profile one kernel under rocprofv3")
    ap.add_argument("--copy-ref", action="store_true", help="run a plain copy of known size (halo_pack of a whole "
                    "16x64x512x512 bf16 interior: 536.9 MB read + 536.9 MB written) to calibrate HBM byte counters")
    ap.add_argument("--unfused", action="store_true", help="store the first stage's unpooled activation (separate conv, pool and "
                    "pool-backward calls) instead of the fused forward + sign mask")
    ap.add_argument("--no-overlap", action="store_true", help="keep every call of the step on one stream (default: the backward-filter "
                    "calls of stages 2.. run on a second stream beside the backward-data chain)")
    ap.add_argument("--calibrate", action="store_true", help="print what this device sustains under the simplest load: a register-only "
                    "bf16 MFMA loop (both tile shapes), a streaming read of 1 GiB and of 64 MiB, and a plain copy")
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--workload", default="cosmoflow", choices=["cosmoflow", "table1", "chain512", "xent", "k5", "shard512", "unet", "late256", "split256", "bn"],
                    help="cosmoflow (default, the metric's configuration); the others print per-call tables of the "
                         "512^3 first-layer shard, the U-Net-shaped level and the 256->256 late layer")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the per-GPU share of the spatially-partitioned path); "
                 "--gpus must be 1")

    import numpy as np
    import torch
    import synth
    from synth import recipes
    import paper_2007_12856_amd as h3d
    from paper_2007_12856_amd.nets import CosmoFlowStack

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    h3d.lib()   # fail loudly if the HIP library is not built
    if args.calibrate:
        ev = lambda: torch.cuda.Event(enable_timing=True)

        def timed(fn, reps):
            fn(0)
            fn(1)
            torch.cuda.synchronize()
            e0, e1 = ev(), ev()
            e0.record()
            for r in range(reps):
                fn(r)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps
        scratch = torch.ones(h3d.probe_mfma_scratch_bytes() // 4, dtype=torch.float32, device="cuda")
        res = {"metric": "calibration", "device": torch.cuda.get_device_name(0)}
        for shape, nm in ((0, "mfma_16x16x32_bf16_tflops"), (1, "mfma_32x32x16_bf16_tflops")):
            fl = []
            ms = timed(lambda r: fl.append(h3d.probe_mfma_bf16(shape, 4096, scratch)), 5)
            res[nm] = round(fl[0] / ms / 1e9, 1)
        sink = torch.zeros(1, dtype=torch.int32, device="cuda")
        big = [torch.ones(1 << 28, dtype=torch.float32, device="cuda") for _ in range(3)]      # 3 x 1 GiB, rotated
        ms = timed(lambda r: h3d.probe_read(big[r % 3], sink), 9)
        res["read_1GiB_gbs"] = round((1 << 30) / ms / 1e6, 1)
        small = [b[i * (1 << 24):(i + 1) * (1 << 24)] for b in big for i in range(16)]             # 48 x 64 MiB, rotated
        ms = timed(lambda r: h3d.probe_read(small[(7 * r) % 48], sink), 48)
        res["read_64MiB_cold_gbs"] = round((1 << 26) / ms / 1e6, 1)
        res["read_64MiB_cold_us"] = round(ms * 1e3, 2)
        del big, small
        t = h3d.Slab(torch.randn((1, 16, 64, 512, 512), device="cuda").to(torch.bfloat16))
        buf = torch.empty_like(t.t)
        ms = timed(lambda r: h3d.halo_pack(t, h3d.FACE_D_LO, 64, buf), 10)
        res["copy_gbs"] = round(2 * t.t.numel() * 2 / ms / 1e6, 1)
        res["published_peaks"] = {"mfma_bf16_tflops": PEAK_MFMA_BF16_TFLOPS, "hbm_gbs": PEAK_HBM_GBS}
        print(json.dumps(res))
        return
    if args.copy_ref:
        t = h3d.Slab(torch.randn((1, 16, 64, 512, 512), device="cuda").to(torch.bfloat16))
        buf = torch.empty_like(t.t)
        for _ in range(args.warmup):
            h3d.halo_pack(t, h3d.FACE_D_LO, 64, buf)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            h3d.halo_pack(t, h3d.FACE_D_LO, 64, buf)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        nbytes = 2 * t.t.numel() * 2
        print(json.dumps({"metric": "copy GB/s", "value": nbytes / ms / 1e6, "unit": "GB/s", "ms": ms, "bytes": nbytes,
                          "kernel": "copy_runs_kernel (halo_pack of a whole interior)"}))
        return
    seed = synth.BASE_SEED if args.seed is None else args.seed
    td = torch.bfloat16 if args.dtype == "bf16" else torch.float32
    if args.workload != "cosmoflow":
        return side_workload(args, seed)

    def dev(a, dt=td):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(dt)

    P = recipes.cosmoflow_params(seed, args.width)
    x, t = recipes.cosmoflow_batch(seed, args.batch, args.width)
    net = CosmoFlowStack(dev(x), dev(t, torch.float32), [(dev(w), dev(b, torch.float32)) for w, b in P["conv"]],
                         [(dev(w), dev(b, torch.float32)) for w, b in P["fc"]], fuse_pool=not args.unfused)
    del P, x
    stream = torch.cuda.current_stream()

    # warm-up; the last warm-up step also times every call on its own to find the dominant one
    for _ in range(max(args.warmup - 1, 0)):
        net.step()
    torch.cuda.synchronize()
    # (two passes back to back, the second one counts: its first call follows a busy GPU like every other call)
    for _ in range(2):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in net.ops]
        for op, (e0, e1) in zip(net.ops, evs):
            e0.record(stream)
            op["fn"]()
            e1.record(stream)
    torch.cuda.synchronize()
    per_call = []
    for op, (e0, e1) in zip(net.ops, evs):
        ms = e0.elapsed_time(e1)
        per_call.append({"name": op["name"], "ms": round(ms, 4),
                         "tflops": round(op["flops"] / ms / 1e9, 2) if op["flops"] and op["name"].startswith("conv") else None,
                         "gbs": round(op["bytes"] / ms / 1e6, 1) if op["bytes"] else None})
    dom = max(range(len(net.ops)), key=lambda i: per_call[i]["ms"])
    if args.only:
        names = [o["name"] for o in net.ops]
        if args.only not in names:
            sys.exit(f"bench.py: --only must be one of {names}")
        dom = names.index(args.only)
        op = net.ops[dom]
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(args.steps):
            op["fn"]()
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        print(json.dumps({"metric": "single call", "kernel": op["name"], "ms": ms, "steps": args.steps,
                          "tflops": op["flops"] / ms / 1e9, "gbs": op["bytes"] / ms / 1e6,
                          "algorithmic_bytes": op["bytes"], "algorithmic_flops": op["flops"]}))
        return

    # the timed steps put the backward-filter calls of stages 2.. on a second stream (joined at the end of every step);
    # the per-call pass above ran everything on one stream so that every call was timed alone
    net.overlap = not args.no_overlap
    net.step()
    torch.cuda.synchronize()
    # timed region: exactly K steps; one HIP-event pair per step around the dominant call
    # (events are recorded on the stream the kernels are launched on)
    dom_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        for i, op in enumerate(net.ops):
            if i == dom:
                dom_ev[k][0].record(stream)
                op["fn"]()
                dom_ev[k][1].record(stream)
            else:
                op["fn"]()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    dom_ms = sum(a.elapsed_time(b) for a, b in dom_ev) / args.steps

    flops = net.conv_flops()
    voxels = args.batch * args.width ** 3
    op = net.ops[dom]
    intensity = op["flops"] / max(op["bytes"], 1)
    if op["flops"] and intensity >= RIDGE:
        roof = {"bound": "mfma", "achieved": op["flops"] / dom_ms / 1e9, "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": op["bytes"] / dom_ms / 1e6, "peak": PEAK_HBM_GBS, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["kernel"] = op["name"]
    roof["ms"] = round(dom_ms, 4)
    roof["algorithmic_bytes"] = op["bytes"]
    roof["algorithmic_flops"] = op["flops"]
    roof["traffic"] = measured_traffic(args.workload, op["name"])

    out = {
        "metric": "conv3d fwd+bwd TFLOP/s", "value": flops / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"CosmoFlow-shaped stack fwd+bwd: N={args.batch} x 4x{args.width}^3, conv 16-32-64-128-256 "
                               f"+ leaky-ReLU + avg-pool, dense 2048-256-4, MSE",
                   "global_batch": args.batch, "input": [4, args.width, args.width, args.width]},
        "voxels_per_s": voxels / (ms_per_step * 1e-3),
        "conv_gflop_per_step": flops / 1e9,
        "pct_of_bf16_mfma_peak": 100.0 * flops / (ms_per_step * 1e-3) / 1e12 / PEAK_MFMA_BF16_TFLOPS,
        "streams": 1 if args.no_overlap else 2,
        "roofline": roof,
        "per_call": per_call,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(seed)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
