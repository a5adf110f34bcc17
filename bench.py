#!/usr/bin/env python3
"""Benchmark of the conv3d hot path on one MI355X: all five benchmark configurations in one run.

A "step" is one pass of the whole hot path of a configuration over one synthetic batch already resident in HBM:
  unet      (configuration 4, the headline: the largest single-GPU configuration, 8.2 TFlop per step) the U-Net-shaped
            level on a 64x256x256 shard of a 256^3 volume, bf16, forward + backward;
  cosmoflow (configuration 2) the CosmoFlow-shaped stack, N=4 x 4x128^3, bf16, forward + backward;
  shard512  (configuration 3) conv 4->16 + leaky-ReLU + avg-pool + the D halo faces on one 8-way depth shard of a 4x512^3 sample;
  late256   (configuration 5) the weight-gradient-bound late layer, N=8, 256->256 channels on 16^3;
  single32  (configuration 1) one fp32 layer, 4->16 channels on 32^3 (the correctness-sized case);
  layer_f32 (beside the five) one fp32 layer of 32->64 channels on 32x128x128: the fp32 matrix-core kernels under load.
For each: W warm-up steps, then EXACTLY K timed steps between two device synchronisations (wall clock), then P >= 10
passes with one HIP-event pair per library call (recorded on the launch stream) whose medians fill the per-call table.

Prints ONE JSON line.  Headline: conv3d fwd+bwd TFLOP/s of the U-Net-shaped level (conv flops by Table I's convention,
2*27*Cin*Cout per output voxel and pass, over the whole step time), voxels/s, `configs` with the same figures, a
per-call table and a per-kernel table for every configuration (fractions of the published peaks AND of the ceilings
measured in this run by the calibration probes), `roofline` for the kernel with the largest total time in the headline
step (HIP events around its calls inside the timed region), and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import ctypes
import hashlib
import json
import os
import statistics
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_BF16_TFLOPS = 2500.0
PEAK_FP32_VALU_TFLOPS = 157.3
PEAK_MFMA_F32_TFLOPS = 157.3          # fp32 tensors: v_mfma_f32_16x16x4_f32
RIDGE = PEAK_MFMA_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
ALL = ["unet", "cosmoflow", "shard512", "late256", "single32"]
# measured in the default run beside the five configurations: an fp32 layer large enough to load the fp32 matrix cores
# (configuration 1, the only fp32 one, is launch-latency-sized)
EXTRA = ["layer_f32"]
OTHERS = ["table1", "chain512", "k5", "split256", "bn", "layer_f32", "faces512"]


# ----------------------------------------------------------------------------------------------- CPU baseline
def cpu_baseline(seed):
    """The oracle, as it stands, on a bounded sample: stage 2 of the CosmoFlow-shaped stack (16->32 channels on 64^3),
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
            "sample": "conv 16->32 ch on 64^3, 4 samples (stage 2 of the CosmoFlow-shaped stack), fwd+bwd_data+bwd_filter, fp64 direct loops",
            "seconds": round(dt, 2), "voxels_per_s": 4 * 64 ** 3 / dt}


# ----------------------------------------------------------------------------------------------- calibration probes
class Probes:
    """ctypes view of libbench_probes.so (bench_probes.hip beside this file; built here when missing)."""

    def __init__(self):
        path = os.path.join(ROOT, "libbench_probes.so")
        if not os.path.exists(path):
            from paper_2007_12856_amd import build
            build.build_probes()
        L = ctypes.CDLL(path)
        P = ctypes.c_void_p
        L.bp_mfma_scratch_bytes.restype = ctypes.c_size_t
        L.bp_mfma_bf16.argtypes = [ctypes.c_int, ctypes.c_int, P, ctypes.c_size_t, ctypes.POINTER(ctypes.c_double), P]
        L.bp_read.argtypes = [P, ctypes.c_size_t, P, ctypes.c_int, ctypes.c_int, ctypes.c_int, P]
        L.bp_write.argtypes = [P, ctypes.c_size_t, ctypes.c_int, P]
        L.bp_copy.argtypes = [P, P, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, P]
        self.L = L

    @staticmethod
    def _stream():
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    def mfma(self, shape, iters, scratch):
        fl = ctypes.c_double(0.0)
        rc = self.L.bp_mfma_bf16(shape, iters, ctypes.c_void_p(scratch.data_ptr()), scratch.numel() * scratch.element_size(),
                                 ctypes.byref(fl), self._stream())
        assert rc == 0, rc
        return fl.value

    def read(self, buf, sink, blocks, unroll=8, contig=0):
        rc = self.L.bp_read(ctypes.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(), ctypes.c_void_p(sink.data_ptr()),
                            blocks, unroll, contig, self._stream())
        assert rc == 0, rc

    def write(self, buf, blocks):
        rc = self.L.bp_write(ctypes.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(), blocks, self._stream())
        assert rc == 0, rc

    def copy(self, src, dst, blocks, unroll=8):
        rc = self.L.bp_copy(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(dst.data_ptr()), src.numel() * src.element_size(),
                            blocks, unroll, self._stream())
        assert rc == 0, rc


def _timed(fn, reps):
    import torch
    fn(0)
    fn(1)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for r in range(reps):
        fn(r)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def calibrate(full=False):
    """What this device sustains under the simplest load: register-only bf16 MFMA loops (both tile shapes), a streaming
    read, write and copy of buffers far larger than the 256 MB last-level cache (rotated).  `full` sweeps grid sizes,
    loads in flight and access order of the read probe."""
    import torch
    pr = Probes()
    res = {"device": torch.cuda.get_device_name(0)}
    scratch = torch.ones(pr.L.bp_mfma_scratch_bytes() // 4 + 4, dtype=torch.float32, device="cuda")
    for shape, nm in ((0, "mfma_16x16x32_bf16_tflops"), (1, "mfma_32x32x16_bf16_tflops")):
        fl = []
        ms = _timed(lambda r: fl.append(pr.mfma(shape, 4096, scratch)), 5)
        res[nm] = round(fl[0] / ms / 1e9, 1)
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    big = [torch.ones(1 << 28, dtype=torch.float32, device="cuda") for _ in range(3)]      # 3 x 1 GiB, rotated
    nb = 1 << 30
    if full:
        sweep = {}
        for blocks in (1024, 2048, 4096, 8192, 16384, 65536):
            for un in (4, 8, 16):
                for contig in (0, 1):
                    ms = _timed(lambda r: pr.read(big[r % 3], sink, blocks, un, contig), 6)
                    sweep[f"blocks{blocks}_inflight{un}_{'contig' if contig else 'stride'}"] = round(nb / ms / 1e6, 1)
        res["read_sweep_gbs"] = sweep
        res["read_1GiB_gbs"] = max(sweep.values())
    else:
        res["read_1GiB_gbs"] = round(max(nb / _timed(lambda r: pr.read(big[r % 3], sink, b, u, 0), 6) / 1e6 for b, u in ((2048, 8), (8192, 8))), 1)
    res["write_1GiB_gbs"] = round(max(nb / _timed(lambda r: pr.write(big[r % 3], b), 6) / 1e6 for b in (2048, 8192)), 1)
    res["copy_1GiB_gbs_read_plus_written"] = round(max(2 * nb / _timed(lambda r: pr.copy(big[r % 3], big[(r + 1) % 3], b, 8), 6) / 1e6
                                                       for b in (2048, 8192)), 1)
    res["published_peaks"] = {"mfma_bf16_tflops": PEAK_MFMA_BF16_TFLOPS, "hbm_gbs": PEAK_HBM_GBS}
    del big
    torch.cuda.empty_cache()
    return res


# ----------------------------------------------------------------------------------------------- workloads
def _randn(gen, shape, dtype, scale=1.0):
    import torch
    return (torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32) * scale).to(dtype)


def _cosmo_field(gen, shape, dtype):
    """log(1 + k), k ~ Poisson(exp(g)), g ~ N(0,1) clipped to +-3: the CosmoFlow stand-in of synth/, drawn on the GPU."""
    import torch
    g = torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32).clamp_(-3.0, 3.0)
    return torch.log1p(torch.poisson(torch.exp(g), generator=gen)).to(dtype)


def _adjacent(lo, hi):
    """The two face buffers of a tensor as halves of one allocation (LO first): the library then packs / unpacks both
    faces in one call."""
    import torch
    both = torch.cat([lo.reshape(-1), hi.reshape(-1)])
    return both[:lo.numel()].view_as(lo), both[lo.numel():].view_as(hi)


def _single_layer(seed, n, cin, cout, d, hw, d_offset, d_global, dtype, field="normal", pool=True, **kw):
    """Harness inputs of one layer on a shard (seeded, drawn on the GPU): x with one halo plane per side, weights
    U[+-sqrt(3/fan_in)], bias U[+-0.1], the gradient slab g ~ N(0,1) with one halo plane per side, pooled gradient."""
    import torch
    import paper_2007_12856_amd as h3d
    from paper_2007_12856_amd.nets import SingleLayer
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    xs = (n, cin, d + 2, hw, hw)
    x = h3d.Slab(_cosmo_field(gen, xs, dtype) if field == "cosmo" else _randn(gen, xs, dtype), 1, 1, d_offset, d_global)
    bound = (3.0 / (27 * cin)) ** 0.5
    w = ((torch.rand((cout, cin, 3, 3, 3), generator=gen, device="cuda") * 2 - 1) * bound).to(dtype)
    b = torch.rand((cout,), generator=gen, device="cuda") * 0.2 - 0.1
    g = h3d.Slab(_randn(gen, (n, cout, d + 2, hw, hw), dtype), 1, 1, d_offset, d_global)
    dp = h3d.Slab(_randn(gen, (n, cout, d // 2, hw // 2, hw // 2), dtype), 0, 0, d_offset // 2, d_global // 2) if pool else None
    return SingleLayer(x, w, b, g, dp, pool=pool, **kw)


def build_workload(name, args, seed):
    """(net, description, network-input voxels per step, storage dtype)."""
    import numpy as np
    import torch
    import synth
    from synth import recipes
    import paper_2007_12856_amd as h3d
    from paper_2007_12856_amd import nets
    bf = torch.bfloat16
    dev = lambda a, dt=bf: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(dt)
    if name == "unet":
        # shapes and distributions of synth.recipes.unet_level_inputs (interior shard, d_offset 64 of 256), drawn on the GPU
        gen = torch.Generator(device="cuda")
        gen.manual_seed(seed)
        P = {k: recipes.conv_params(seed, 310 + 2 * i, ci, co, taps=8 if k == "up" else 27, transposed=(k == "up"))
             for i, (k, (ci, co)) in enumerate(recipes.UNET_WIDTHS.items())}
        x = _randn(gen, (1, 1, 68, 256, 256), bf)
        dout = _randn(gen, (1, 64, 64, 256, 256), bf)
        spec = {"p": (64, 2, 2, True), "cat": (128, 1, 1, True), "g6": (64, 1, 1, False), "g4": (128, 1, 2, False),
                "g3": (64, 1, 2, False), "g2": (64, 1, 1, False), "g1": (32, 1, 1, False)}
        faces = {}
        for k, (c, width, level, nonneg) in spec.items():
            pair = [_randn(gen, (1, c, width, 256 // level, 256 // level), bf) for _ in range(2)]
            faces[k] = _adjacent(*(torch.relu(f) if nonneg else f for f in pair))
        net = nets.UNetLevel(h3d.Slab(x, 2, 2, 64, 256), {k: (dev(w), dev(b, torch.float32)) for k, (w, b) in P.items()}, dout, faces)
        return net, ("U-Net-shaped level on an interior 64x256x256 shard of a 1-channel 256^3 volume (2-voxel halo), bf16: conv 1-32-64, "
                     "max-pool, conv 64-64-128, transposed conv 128-64, concat, conv 128-64, ReLU; fwd+bwd"), 64 * 256 * 256, "bf16"
    if name == "cosmoflow":
        td = bf if args.dtype == "bf16" else torch.float32
        P = recipes.cosmoflow_params(seed, args.width)
        gen = torch.Generator(device="cuda")
        gen.manual_seed(seed)
        x = _cosmo_field(gen, (args.batch, 4, args.width, args.width, args.width), td)       # the recipe of synth.recipes.cosmoflow_batch, on the GPU
        t = torch.rand((args.batch, 4), generator=gen, device="cuda") * 2 - 1
        net = nets.CosmoFlowStack(x, t, [(dev(w, td), dev(b, torch.float32)) for w, b in P["conv"]],
                                  [(dev(w, td), dev(b, torch.float32)) for w, b in P["fc"]], fuse_pool=not args.unfused)
        net.overlap = not args.no_overlap
        return net, (f"CosmoFlow-shaped stack: N={args.batch} x 4x{args.width}^3, conv 16-32-64-128-256 + leaky-ReLU + avg-pool, "
                     f"dense 2048-256-4, MSE; fwd+bwd; {2 if net.overlap else 1} streams"), args.batch * args.width ** 3, args.dtype
    if name == "shard512":
        net = _single_layer(seed, 1, 4, 16, 64, 512, 64, 512, bf, field="cosmo", fuse_pool=not args.unfused)
        return net, ("one interior 8-way depth shard of a 4x512^3 sample: 4x66x512x512 bf16, conv 4->16 + leaky-ReLU + avg-pool "
                     + ("(three separate passes)" if args.unfused else "(one fused call, sign mask for the backward pass)") +
                     ", bwd-data / bwd-filter, D halo faces packed and unpacked"), 64 * 512 * 512, "bf16"
    if name == "faces512":
        # the H and W faces (1 and 2 voxels wide, both ends) of the same shard's 16-channel activation gradient
        net = _single_layer(seed, 1, 4, 16, 64, 512, 64, 512, bf, field="cosmo", faces_hw=True)
        net.ops = [o for o in net.ops if o["name"].startswith("face_")]
        return net, ("H and W faces of a 16x66x512x512 bf16 activation gradient (a partitioning in H or W as well): pack and unpack, "
                     "1 and 2 voxels wide, both ends"), 64 * 512 * 512, "bf16"
    if name == "late256":
        net = _single_layer(seed, 8, 256, 256, 16, 16, 0, 16, bf, pool=False, halo_ops=False)       # whole 16^3 volumes: no faces
        return net, "weight-gradient-bound late layer: N=8, 256->256 channels, 16^3, bf16, fwd / bwd-data / bwd-filter", 8 * 16 ** 3, "bf16"
    if name == "single32":
        net = _single_layer(seed, 1, 4, 16, 32, 32, 0, 32, torch.float32, pool=False, halo_ops=False)
        return net, "single layer, fp32: N=1, 4->16 channels, 32^3, bias + leaky-ReLU, fwd / bwd-data / bwd-filter", 32 ** 3, "f32"
    if name == "layer_f32":
        net = _single_layer(seed, 1, 32, 64, 32, 128, 0, 32, torch.float32, pool=False, halo_ops=False)
        return net, "one layer in the paper's precision: fp32 storage and arithmetic, 32->64 channels on 32x128x128, fwd / bwd-data / bwd-filter", 32 * 128 * 128, "f32"
    if name == "split256":
        net = _single_layer(seed, 1, 64, 64, 32, 256, 32, 256, bf, pool=False, split=True)
        return net, "one 8-way depth shard of a 64-channel 256^3 sample: conv 64->64 whole, and as main planes + two 1-plane strips", 32 * 256 * 256, "bf16"
    if name == "bn":
        gen = torch.Generator(device="cuda")
        gen.manual_seed(seed)
        net = nets.BatchNormLayer(h3d.Slab(_randn(gen, (4, 16, 128, 128, 128), bf)), h3d.Slab(_randn(gen, (4, 16, 128, 128, 128), bf)))
        return net, "local batch-normalisation passes on the first convolution's output: 4 x 16 x 128^3 bf16", 4 * 128 ** 3, "bf16"
    if name == "table1":
        channels, strides, pools, flat_w = recipes.table1_layout(args.width)
        P = recipes.cosmoflow_params(seed, args.width, channels, recipes.COSMO_FC, flat_w)
        x, t = recipes.cosmoflow_batch(seed, args.batch, args.width)
        net = nets.CosmoFlowStack(dev(x), dev(t, torch.float32), [(dev(w), None) for w, _ in P["conv"]],
                                  [(dev(w), dev(b, torch.float32)) for w, b in P["fc"]], fuse_pool=not args.unfused,
                                  strides=strides, pools=pools)
        net.overlap = not args.no_overlap
        return net, (f"network of Table I for {args.width}^3 inputs, N={args.batch}: conv 16-32-64-128(stride 2)-256-256-256, no conv biases, "
                     f"leaky-ReLU, avg-pool, dense 2048-256-4, MSE; fwd+bwd; {net.conv_flops() / args.batch / 1e9:.2f} conv GFlop per sample"), \
            args.batch * args.width ** 3, "bf16"
    if name == "chain512":
        x, conv, dout, faces = recipes.shard_chain_inputs(seed, 512, 64, 64, 512, n=args.batch)
        net = nets.CosmoFlowShardChain(h3d.Slab(dev(x), 1, 1, 64, 512), [(dev(w), None) for w, _ in conv], dev(dout),
                                       {k: _adjacent(dev(lo), dev(hi)) for k, (lo, hi) in faces.items()}, fuse_pool=not args.unfused)
        return net, (f"conv1-pool1 .. conv3-pool3 of Table I's 512^3 network on one interior shard of an 8-way depth partition "
                     f"(N={args.batch} x 4x(64+2)x512x512 bf16), halo faces packed and unpacked per stage, fwd+bwd"), args.batch * 64 * 512 * 512, "bf16"
    if name == "k5":
        return _k5_workload(seed), "5x5x5 convolution 32->32, 32-plane interior shard (+2 halo planes per side) of a 128^3 volume, bf16, three passes", \
            32 * 128 * 128, "bf16"
    raise SystemExit(f"bench.py: unknown workload {name}")


def _k5_workload(seed):
    import torch
    import paper_2007_12856_amd as h3d
    bf = torch.bfloat16

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
    return _K5()


# ----------------------------------------------------------------------------------------------- measurement
def lib_source_hash():
    """sha16 over the HIP sources of the library: a stored traffic figure only counts for the code it was measured on."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2007_12856_amd", "csrc")
    for f in sorted(os.listdir(d)):
        if f.endswith((".hip", ".h")):
            h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` in `workload`, from two `rocprofv3 --pmc` runs (FETCH_SIZE, then WRITE_SIZE) scaled by
    the plain-copy factors: the line 'TRAFFIC <workload> <kernel> <bytes per launch> <source hash>' of profiles/hbm_traffic.txt
    (commands and raw counter values in that file).  None when there is no line for this kernel or when the library's sources
    have changed since it was measured."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    cur = lib_source_hash()
    for line in open(path):
        f = line.split()
        if len(f) == 5 and f[0] == "TRAFFIC" and f[1] == workload and f[2] == kernel and f[4] == cur:
            return int(f[3])
    return None


def fractions(flops, nbytes, ms, ceil, dtype="bf16"):
    """TFLOP/s, GB/s and their fractions of the published peaks and of the ceilings measured by the probes.  The matrix-core
    peak is that of the tensors' own type (bf16: 2500 TFLOP/s, fp32: 157.3); the measured ceiling exists for bf16 only."""
    out = {}
    peak = PEAK_MFMA_F32_TFLOPS if dtype == "f32" else PEAK_MFMA_BF16_TFLOPS
    if flops:
        tf = flops / ms / 1e9
        out.update(tflops=round(tf, 2), mfma_frac=round(tf / peak, 4))
        if ceil and dtype != "f32":
            out["mfma_frac_of_measured"] = round(tf / ceil["mfma_32x32x16_bf16_tflops"], 4)
    if nbytes:
        gb = nbytes / ms / 1e6
        out.update(gbs=round(gb, 1), hbm_frac=round(gb / PEAK_HBM_GBS, 4))
        if ceil:
            out["hbm_frac_of_measured"] = round(gb / ceil["copy_1GiB_gbs_read_plus_written"], 4)
    if flops or nbytes:
        out["bound"] = "mfma" if flops and flops / max(nbytes, 1) >= peak * 1e12 / (PEAK_HBM_GBS * 1e9) else "hbm"
    return out


def run_workload(name, args, seed, ceil, steps, warmup, passes, events_for=None):
    """Warm-up, K timed steps (wall clock between two synchronisations), `passes` per-call passes (HIP events on the launch
    stream, medians).  Returns the result dict; `events_for(kernel_table)` (headline only) picks the kernel whose calls get an
    event pair inside the timed region."""
    import torch
    import paper_2007_12856_amd as h3d
    t_build = time.perf_counter()
    net, label, voxels, dtype = build_workload(name, args, seed)
    t_build = time.perf_counter() - t_build
    stream = torch.cuda.current_stream()
    ev = lambda: torch.cuda.Event(enable_timing=True)
    overlap = getattr(net, "overlap", False)
    for _ in range(max(warmup, 1)):
        net.step()
    torch.cuda.synchronize()
    # which kernel does each call run (asked of the library after the call)
    kernels = []
    for o in net.ops:
        o["fn"]()
        kernels.append(h3d.h3d_last_kernel() if (o["flops"] or o["bytes"]) else "")
    torch.cuda.synchronize()

    def per_call_pass():
        evs = []
        for o in net.ops:
            e0, e1 = ev(), ev()
            e0.record(stream)
            o["fn"]()
            e1.record(stream)
            evs.append((e0, e1))
        torch.cuda.synchronize()
        return [a.elapsed_time(b) for a, b in evs]

    # the per-call passes run on ONE stream so that every call is timed alone
    if overlap:
        net.overlap = False
    per_call_pass()
    samples = [per_call_pass() for _ in range(passes)]
    med = [statistics.median(s[i] for s in samples) for i in range(len(net.ops))]
    if overlap:
        net.overlap = True
        net.step()
        torch.cuda.synchronize()
    # kernel table: calls grouped by the kernel the library ran for them
    groups = {}
    for o, k, ms in zip(net.ops, kernels, med):
        if not k:
            continue
        g = groups.setdefault(k, {"kernel": k, "calls": [], "ms": 0.0, "flops": 0, "bytes": 0})
        g["calls"].append(o["name"])
        g["ms"] += ms
        g["flops"] += o["flops"]
        g["bytes"] += o["bytes"]
    ktable = sorted(groups.values(), key=lambda g: -g["ms"])
    dom = events_for(ktable) if events_for else None
    dom_idx = [i for i, k in enumerate(kernels) if dom and k == dom["kernel"]]
    dom_ev = []
    # ---- timed region: exactly K steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        if dom_idx:
            for i, o in enumerate(net.ops):
                if i in dom_idx:
                    e0, e1 = ev(), ev()
                    e0.record(stream)
                    o["fn"]()
                    e1.record(stream)
                    dom_ev.append((i, e0, e1))
                else:
                    o["fn"]()
        else:
            net.step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    flops = net.conv_flops()
    per_call = []
    for o, k, ms in zip(net.ops, kernels, med):
        row = {"name": o["name"], "ms": round(ms, 4)}
        if k:
            row["kernel"] = k
        row.update(fractions(o["flops"], o["bytes"], ms, ceil, dtype))
        per_call.append(row)
    for g in ktable:
        g.update(fractions(g["flops"], g["bytes"], g["ms"], ceil, dtype))
        g["ms"] = round(g["ms"], 4)
        g["share_of_step"] = round(g["ms"] / sum(med), 4)
    res = {"workload": label, "dtype": dtype, "ms_per_step": round(ms_per_step, 4), "ms_per_step_sum_of_calls": round(sum(med), 4),
           "conv_gflop_per_step": round(flops / 1e9, 2), "tflops": round(flops / ms_per_step / 1e9, 2),
           "mfma_frac": round(flops / ms_per_step / 1e9 / (PEAK_MFMA_F32_TFLOPS if dtype == "f32" else PEAK_MFMA_BF16_TFLOPS), 4), "voxels_per_s": round(voxels / (ms_per_step * 1e-3), 1),
           "steps": steps, "passes": passes, "setup_s": round(t_build, 1), "per_kernel": ktable, "per_call": per_call}
    if dom:
        per_step = {}
        for i, a, b in dom_ev:
            per_step.setdefault(i, []).append(a.elapsed_time(b))
        launches = len(dom_idx)
        ms_total = sum(sum(v) / len(v) for v in per_step.values())          # mean over the K steps, summed over the kernel's calls
        res["dominant"] = {"kernel": dom["kernel"], "calls": [net.ops[i]["name"] for i in dom_idx], "launches_per_step": launches,
                           "ms_per_launch": ms_total / launches, "flops_per_launch": dom["flops"] / launches, "bytes_per_launch": dom["bytes"] / launches}
    del net
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--passes", type=int, default=11, help="per-call passes whose medians fill the tables (at least 10)")
    ap.add_argument("--batch", type=int, default=4)
    ap.add_argument("--width", type=int, default=128)
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "f32"], help="storage type of the cosmoflow workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-calibration", action="store_true", help="skip the probes (fractions of the measured ceilings are then absent)")
    ap.add_argument("--only", default=None, help="with --workload NAME: after warm-up, run only this call of the step (name as in per_call) "
                    "--steps times; used to profile one kernel under rocprofv3")
    ap.add_argument("--copy-ref", action="store_true", help="run a plain copy of known size (halo_pack of a whole "
                    "16x64x512x512 bf16 interior: 536.9 MB read + 536.9 MB written) to calibrate HBM byte counters")
    ap.add_argument("--unfused", action="store_true", help="cosmoflow / table1 / chain512 / shard512: store the first stage's unpooled activation "
                    "(separate conv, pool and pool-backward calls) instead of the fused forward + sign mask")
    ap.add_argument("--no-overlap", action="store_true", help="cosmoflow / table1: keep every call of the step on one stream (default: the "
                    "backward-filter calls of the late stages run on a second stream beside the backward-data chain)")
    ap.add_argument("--calibrate", action="store_true", help="print only what this device sustains under the simplest load (with a sweep of "
                    "the read probe's grid size, loads in flight and access order)")
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--workload", default="all", choices=["all"] + ALL + OTHERS,
                    help="all (default): the five benchmark configurations, headline on the U-Net-shaped level; one name: that workload alone")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the per-GPU share of the spatially-partitioned path); "
                 "--gpus must be 1")

    import torch
    import synth
    import paper_2007_12856_amd as h3d

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    h3d.lib()   # fail loudly if the HIP library is not built
    seed = synth.BASE_SEED if args.seed is None else args.seed
    if args.calibrate:
        print(json.dumps({"metric": "calibration", **calibrate(full=True)}))
        return
    if args.copy_ref:
        t = h3d.Slab(torch.randn((1, 16, 64, 512, 512), device="cuda").to(torch.bfloat16))
        buf = torch.empty_like(t.t)
        ms = _timed(lambda r: h3d.halo_pack(t, h3d.FACE_D_LO, 64, buf), args.steps)
        nbytes = 2 * t.t.numel() * 2
        print(json.dumps({"metric": "copy GB/s", "value": nbytes / ms / 1e6, "unit": "GB/s", "ms": ms, "bytes": nbytes,
                          "kernel": "copy_runs_kernel (halo_pack of a whole interior)"}))
        return
    if args.only:
        if args.workload == "all":
            sys.exit("bench.py: --only needs --workload NAME")
        net, label, _, _ = build_workload(args.workload, args, seed)
        if hasattr(net, "overlap"):
            net.overlap = False
        sel = [o for o in net.ops if o["name"] == args.only]
        if not sel:
            sys.exit(f"bench.py: --only must be one of {[o['name'] for o in net.ops]}")
        for _ in range(args.warmup):
            net.step()
        torch.cuda.synchronize()
        stream = torch.cuda.current_stream()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(args.steps):
            sel[0]["fn"]()
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        print(json.dumps({"metric": "single call", "call": args.only, "kernel": h3d.h3d_last_kernel(), "ms": ms, "steps": args.steps,
                          "tflops": sel[0]["flops"] / ms / 1e9, "gbs": sel[0]["bytes"] / ms / 1e6, "algorithmic_bytes": sel[0]["bytes"],
                          "algorithmic_flops": sel[0]["flops"], "config": {"workload": label}}))
        return

    ceil = None if args.no_calibration else calibrate()
    halo_rate = None
    if args.workload == "all":
        # one batched halo call of a size where the copy is not launch-bound (Sec. III-A packing kernels): the two lower
        # halo planes of 8 samples x 32 channels x 512 x 512, 134 MB read + 134 MB written
        t = h3d.Slab(torch.randn((8, 32, 6, 512, 512), device="cuda").to(torch.bfloat16), 2, 2, 8, 64)
        buf = torch.empty((8 * 32 * 2 * 512 * 512,), dtype=torch.bfloat16, device="cuda")
        ms = _timed(lambda r: h3d.halo_pack(t, h3d.FACE_D_LO, 2, buf), 20)
        nbytes = 2 * buf.numel() * 2
        halo_rate = {"call": "halo_pack, 2 planes of 8 x 32 x 512 x 512 bf16", "bytes_read_plus_written": nbytes, "ms": round(ms, 4),
                     "gbs": round(nbytes / ms / 1e6, 1), "hbm_frac": round(nbytes / ms / 1e6 / PEAK_HBM_GBS, 4)}
        del t, buf
    names = ALL + EXTRA if args.workload == "all" else [args.workload]
    head = names[0]
    passes = max(args.passes, 10)
    results = {}
    for nm in names:
        results[nm] = run_workload(nm, args, seed, ceil, args.steps, args.warmup, passes,
                                   events_for=(lambda kt: kt[0] if kt else None) if nm == head else None)
    H = results[head]
    out = {
        "metric": "conv3d fwd+bwd TFLOP/s", "value": H["tflops"], "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": H["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": H["dtype"], "data": "synthetic",
        "config": {"workload": H["workload"], "name": head},
        "voxels_per_s": H["voxels_per_s"], "conv_gflop_per_step": H["conv_gflop_per_step"],
        ("pct_of_fp32_mfma_peak" if H["dtype"] == "f32" else "pct_of_bf16_mfma_peak"): round(100.0 * H["mfma_frac"], 2),
    }
    f32 = H["dtype"] == "f32"
    mfma_peak = PEAK_MFMA_F32_TFLOPS if f32 else PEAK_MFMA_BF16_TFLOPS
    d = H.get("dominant")
    if d:
        ms = d["ms_per_launch"]
        if d["flops_per_launch"] and d["flops_per_launch"] / max(d["bytes_per_launch"], 1) >= mfma_peak * 1e12 / (PEAK_HBM_GBS * 1e9):
            roof = {"bound": "mfma", "achieved": d["flops_per_launch"] / ms / 1e9, "peak": mfma_peak, "unit": "TFLOP/s"}
            if ceil and not f32:
                roof["frac_of_measured_ceiling"] = roof["achieved"] / ceil["mfma_32x32x16_bf16_tflops"]
        else:
            roof = {"bound": "hbm", "achieved": d["bytes_per_launch"] / ms / 1e6, "peak": PEAK_HBM_GBS, "unit": "GB/s"}
            if ceil:
                roof["frac_of_measured_ceiling"] = roof["achieved"] / ceil["copy_1GiB_gbs_read_plus_written"]
        roof["frac"] = roof["achieved"] / roof["peak"]
        roof.update(kernel=d["kernel"], calls=d["calls"], launches_per_step=d["launches_per_step"], ms=round(ms, 4),
                    algorithmic_bytes=d["bytes_per_launch"], algorithmic_flops=d["flops_per_launch"],
                    traffic=measured_traffic(head, d["kernel"]))
        out["roofline"] = roof
    if ceil:
        out["measured_ceilings"] = ceil
    if halo_rate:
        out["halo_batched"] = halo_rate
    out["configs"] = results
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(seed)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
