"""Call sequences of the two network shapes over the C-ABI binding (no arithmetic here: every
step is one library call; buffers are allocated once, a step allocates nothing).

CosmoFlowStack: conv3d 3x3x3 + leaky-ReLU + 2x2x2 average pooling stages, flatten, three
fully-connected layers, MSE loss (the network of Table I, Sec. IV, in the 5-stage shape the
benchmark configuration names), forward and backward (BD and BF of every layer, Sec. III-C).
"""
from __future__ import annotations

import torch

from . import (ACT_LEAKY, ACT_NONE, POOL_AVG, Slab, Workspace, conv3d_bwd_data, conv3d_bwd_filter, conv3d_fwd,
               conv3d_fwd_pool, conv3d_s2_bwd_data, conv3d_s2_bwd_filter, conv3d_s2_fwd, dense_bwd, dense_fwd, mse_fwd_bwd, pool3d_bwd, pool3d_bwd_act, pool3d_bwd_mask, pool3d_fwd, pool3d_fwd_mask)


def face_pair(t: "Slab", width: int):
    """Two face buffers of `t` (LO, HI) that are the halves of ONE allocation, so that both faces can go through a single
    halo_pack / halo_unpack call (FACE_D_BOTH)."""
    from . import halo_bytes
    k = halo_bytes(t, width) // t.t.element_size()
    both = torch.empty(2 * k, dtype=t.t.dtype, device=t.t.device)
    return both[:k], both[k:]


def _adjacent(lo, hi) -> bool:
    return (lo is not None and hi is not None and lo.is_contiguous() and hi.is_contiguous() and lo.numel() == hi.numel()
            and lo.data_ptr() + lo.numel() * lo.element_size() == hi.data_ptr())


def pack_faces(t: "Slab", width: int, lo, hi):
    """The two depth faces of t's interior into lo / hi: one call when the two buffers are adjacent in memory."""
    from . import FACE_D_BOTH, FACE_D_HI, FACE_D_LO, halo_pack
    if _adjacent(lo, hi):
        halo_pack(t, FACE_D_BOTH, width, lo)
    else:
        halo_pack(t, FACE_D_LO, width, lo)
        halo_pack(t, FACE_D_HI, width, hi)


def unpack_faces(lo, hi, t: "Slab", width: int):
    """lo / hi (None: zero fill, the global boundary) into the two halos of t: one call when the two buffers are adjacent
    in memory, or both are None."""
    from . import FACE_D_BOTH, FACE_D_HI, FACE_D_LO, halo_unpack
    if _adjacent(lo, hi) or (lo is None and hi is None):
        halo_unpack(lo, t, FACE_D_BOTH, width)
    else:
        halo_unpack(lo, t, FACE_D_LO, width)
        halo_unpack(hi, t, FACE_D_HI, width)


class CosmoFlowStack:
    def __init__(self, x: torch.Tensor, target: torch.Tensor, conv_params, fc_params, alpha: float = 0.01, fuse_pool: bool = False,
                 strides=None, pools=None):
        """x [N,C,D,H,W] device tensor; conv_params/fc_params: lists of (w, bias) device tensors
        (w in x's dtype, bias fp32 or None: the paper's variant drops the convolution biases, Sec. IV);
        target fp32 [N, nout].  strides[i] in (1, 2): stride of convolution i (Table I: the fourth has 2);
        pools[i]: whether a 2x2x2 average pooling follows it (Table I: the last layers of the small inputs
        have none, their volume is already 2^3).  Defaults: stride 1, pooling everywhere."""
        self.alpha = alpha
        self.ws = Workspace()
        # backward-filter of a layer and its backward-data only share their input g: with `overlap` set, the
        # backward-filter calls of the small late layers (latency-bound, they leave most of the chip idle) go to a
        # second HIP stream (default priority) with a workspace of their own and are joined at the end of the step
        self.overlap = False
        self._pending = False
        # measured: the backward-filter calls of stages 3.. beside the backward-data chain save 6 % of the step; the
        # second stage's call fills the chip by itself, and the first stage's calls are HBM-bound and run alone, its
        # backward-data first so that the side stream has drained when the longest call of the step starts
        self.side_min = 2
        self.bd_first = True
        self.side = None
        dt, dev = x.dtype, x.device
        nconv = len(conv_params)
        self.strides = list(strides) if strides is not None else [1] * nconv
        self.pools = list(pools) if pools is not None else [True] * nconv
        # fuse_pool: stages whose convolution has a fused forward (first layer: Cin <= 4) never store the unpooled
        # activation: the forward writes the pooled tensor and a sign mask, the backward reads the mask
        self.fused = [bool(fuse_pool) and dt == torch.bfloat16 and w.shape[1] <= 4 and w.shape[0] <= 32 and self.strides[i] == 1
                      and self.pools[i] for i, (w, _) in enumerate(conv_params)]
        self.x = Slab(x)
        self.target = target
        self.conv, self.fc = conv_params, fc_params
        n = x.shape[0]
        self.z, self.p, self.mask, self.g, self.dp = [], [], [], [], []
        cur = self.x
        for i, (w, _) in enumerate(conv_params):
            st = self.strides[i]
            zd, zh, zw = cur.d // st, (cur.t.shape[3] + st - 1) // st, (cur.t.shape[4] + st - 1) // st
            fused = self.fused[i] and zd % 2 == 0 and zh % 2 == 0 and zw % 16 == 0
            self.fused[i] = fused
            zshape = (n, w.shape[0], zd, zh, zw)
            z = None if fused else Slab(torch.empty(zshape, dtype=dt, device=dev))
            # stored activations that are pooled: the pooling forward also writes their sign mask (it reads them anyway), and
            # the pooling backward takes the mask instead of reading the activation again
            masked = (fused or (bool(fuse_pool) and dt == torch.bfloat16 and self.pools[i] and zd % 2 == 0 and zh % 2 == 0 and zw % 16 == 0))
            self.mask.append(torch.empty((n * w.shape[0] * zd * zh * zw // 8,), dtype=torch.uint8, device=dev) if masked else None)
            # g: gradient at the convolution's output; after a pooling it is already multiplied by the activation
            # derivative (pooling backward and activation backward are one call), else it is the raw dz
            self.g.append(Slab(torch.empty(zshape, dtype=dt, device=dev)))
            if self.pools[i]:
                p = Slab(torch.empty((n, w.shape[0], zd // 2, zh // 2, zw // 2), dtype=dt, device=dev))
                self.dp.append(Slab(torch.empty_like(p.t)))
            else:
                p = None
                self.dp.append(None)
            self.z.append(z)
            self.p.append(p)
            cur = p if p is not None else z
        self.out = [p if p is not None else z for p, z in zip(self.p, self.z)]            # what the next layer reads
        self.dout = [dp if dp is not None else g for dp, g in zip(self.dp, self.g)]       # where its gradient arrives
        self.flat = cur.t.view(n, -1)
        self.y = [torch.empty((n, w.shape[0]), dtype=dt, device=dev) for w, _ in fc_params]
        self.loss = torch.empty((1,), dtype=torch.float32, device=dev)
        # gradients
        self.dy = [torch.empty_like(y) for y in self.y]
        self.dfc = [(torch.empty(w.shape, dtype=torch.float32, device=dev), torch.empty(b.shape, dtype=torch.float32, device=dev))
                    for w, b in fc_params]
        self.dx = Slab(torch.empty_like(x))
        self.dconv = [(torch.empty(w.shape, dtype=torch.float32, device=dev),
                       None if b is None else torch.empty(b.shape, dtype=torch.float32, device=dev)) for w, b in conv_params]

        self._build_ops()

    # ------------------------------------------------------------------ the step as a list of library calls
    def _op(self, name, fn, flops=0, nbytes=0):
        self.ops.append({"name": name, "fn": fn, "flops": int(flops), "bytes": int(nbytes)})

    def _build_ops(self):
        """Each entry is ONE library call with its algorithmic work: conv flops = 2*27*Cin*Cout per
        output voxel (Table I's convention); bytes = every input and output tensor once."""
        self.ops = []
        es = self.x.t.element_size()
        al, ws = self.alpha, self.ws
        nconv, last = len(self.conv), len(self.fc) - 1
        cur = self.x
        for i, (w, b) in enumerate(self.conv):
            z, p = self.z[i], self.p[i]
            zvox = self.g[i].t.numel() // w.shape[0]
            fl = 2 * 27 * w.shape[1] * w.shape[0] * zvox
            if self.fused[i]:
                zshape, mask = tuple(self.g[i].t.shape), self.mask[i]
                self._op(f"conv{i + 1}_fwd_pool", lambda cur=cur, w=w, b=b, zshape=zshape, p=p, mask=mask: conv3d_fwd_pool(
                    cur, w, b, zshape, p, mask, ACT_LEAKY, al, ws), fl, (cur.t.numel() + p.t.numel() + w.numel()) * es + mask.numel())
            else:
                io = (cur.t.numel() + z.t.numel() + w.numel()) * es
                fwd = conv3d_s2_fwd if self.strides[i] == 2 else conv3d_fwd
                self._op(f"conv{i + 1}_fwd", lambda cur=cur, w=w, b=b, z=z, fwd=fwd: fwd(cur, w, b, z, ACT_LEAKY, al, ws), fl, io)
                if p is not None and self.mask[i] is not None:
                    mask = self.mask[i]
                    self._op(f"pool{i + 1}_fwd", lambda z=z, p=p, mask=mask: pool3d_fwd_mask(z, p, mask), 0,
                             (z.t.numel() + p.t.numel()) * es + mask.numel())
                elif p is not None:
                    self._op(f"pool{i + 1}_fwd", lambda z=z, p=p: pool3d_fwd(z, p, POOL_AVG), 0, (z.t.numel() + p.t.numel()) * es)
            cur = self.out[i]
        h = self.flat
        for i, (w, b) in enumerate(self.fc):
            y = self.y[i]
            act = ACT_NONE if i == last else ACT_LEAKY
            self._op(f"fc{i + 1}_fwd", lambda h=h, w=w, b=b, y=y, act=act: dense_fwd(h, w, b, y, act, al),
                     2 * h.shape[0] * w.numel(), (w.numel() + h.numel() + y.numel()) * es)
            h = y
        self.n_fwd_ops = len(self.ops)
        self._op("mse", lambda: mse_fwd_bwd(self.y[last], self.target, self.loss, self.dy[last]))
        for i in range(last, -1, -1):
            xin = self.flat if i == 0 else self.y[i - 1]
            dxin = self.dout[-1].t.view(xin.shape) if i == 0 else self.dy[i - 1]
            w = self.fc[i][0]
            act = ACT_NONE if i == last else ACT_LEAKY
            # two independent halves: dx on the current stream (the chain continues with it), dw / db beside it
            self._op(f"fc{i + 1}_bwd", lambda xin=xin, w=w, i=i, dxin=dxin, act=act: (
                dense_bwd(xin, w, self.y[i], self.dy[i], dxin, None, None, act, al),
                self._on_side(lambda _ws: dense_bwd(xin, w, self.y[i], self.dy[i], None, self.dfc[i][0], self.dfc[i][1], act, al))),
                4 * xin.shape[0] * w.numel(), w.numel() * es + w.numel() * 4)
        for i in range(nconv - 1, -1, -1):
            w = self.conv[i][0]
            z, g, dp = self.z[i], self.g[i], self.dp[i]
            xin = self.x if i == 0 else self.out[i - 1]
            dxin = self.dx if i == 0 else self.dout[i - 1]
            fl = 2 * 27 * w.shape[1] * g.t.numel()
            zb, actb = None, ACT_NONE
            if dp is not None and self.mask[i] is not None:
                # pooling backward and activation backward in one pass; BF and BD then run unmasked on g
                mask = self.mask[i]
                self._op(f"pool{i + 1}_bwd_mask", lambda dp=dp, mask=mask, g=g: pool3d_bwd_mask(dp, mask, g, ACT_LEAKY, al), 0,
                         (dp.t.numel() + g.t.numel()) * es + mask.numel())
            elif dp is not None:
                self._op(f"pool{i + 1}_bwd_act", lambda dp=dp, z=z, g=g: pool3d_bwd_act(dp, None, z, g, POOL_AVG, ACT_LEAKY, al), 0,
                         (dp.t.numel() + z.t.numel() + g.t.numel()) * es)
            else:
                zb, actb = z, ACT_LEAKY          # no pooling: g is the raw dz, BF and BD apply the activation derivative from z
            bf = conv3d_s2_bwd_filter if self.strides[i] == 2 else conv3d_bwd_filter
            bd = conv3d_s2_bwd_data if self.strides[i] == 2 else conv3d_bwd_data
            def add_bd():
                self._op(f"conv{i + 1}_bwd_data", lambda g=g, w=w, dxin=dxin, bd=bd, zb=zb, actb=actb: bd(g, zb, w, dxin, actb, al, ws),
                         fl, (g.t.numel() + dxin.t.numel() + w.numel()) * es)

            if i >= self.side_min:
                self._op(f"conv{i + 1}_bwd_filter", lambda xin=xin, g=g, i=i, bf=bf, zb=zb, actb=actb: self._on_side(
                    lambda wsx: bf(xin, g, zb, self.dconv[i][0], self.dconv[i][1], actb, al, wsx)), fl,
                    (xin.t.numel() + g.t.numel()) * es + w.numel() * 4)
                add_bd()
            else:
                if self.bd_first:
                    add_bd()
                self._op(f"conv{i + 1}_bwd_filter", lambda xin=xin, g=g, i=i, bf=bf, zb=zb, actb=actb: bf(
                    xin, g, zb, self.dconv[i][0], self.dconv[i][1], actb, al, ws), fl,
                    (xin.t.numel() + g.t.numel()) * es + w.numel() * 4)
                if not self.bd_first:
                    add_bd()
        self._op("join", self._join)

    def _on_side(self, call):
        """Run `call(workspace)` on the side stream, ordered after what the current stream holds at this moment."""
        if not self.overlap:
            return call(self.ws)
        if self.side is None:
            self.side = torch.cuda.Stream()           # default priority
            self.ws_side = Workspace()
            self._fork, self._joined = torch.cuda.Event(), torch.cuda.Event()
        self._fork.record(torch.cuda.current_stream())
        self.side.wait_event(self._fork)
        with torch.cuda.stream(self.side):
            call(self.ws_side)
        self._pending = True

    def _join(self):
        """The current stream waits for the side stream (the next forward overwrites what its calls read)."""
        if self._pending:
            self._joined.record(self.side)
            torch.cuda.current_stream().wait_event(self._joined)
            self._pending = False

    def forward(self):
        for op in self.ops[:self.n_fwd_ops]:
            op["fn"]()
        return self.y[-1]

    def backward(self):
        for op in self.ops[self.n_fwd_ops:]:
            op["fn"]()

    def backward_after_loss(self):
        """Backward from a loss gradient already present in self.dy[-1] (skips the MSE call)."""
        for op in self.ops[self.n_fwd_ops + 1:]:
            op["fn"]()

    def step(self):
        for op in self.ops:
            op["fn"]()

    def conv_flops(self) -> int:
        return sum(op["flops"] for op in self.ops if op["name"].startswith("conv"))


class UNetLevel:
    """One encoder/decoder level of a 3D U-Net on a depth shard (Sec. II-C, III-A): two 3x3x3
    conv+ReLU (the first also produces its output's halo plane from the 2-plane input halo), 2x2x2
    max-pool, two conv+ReLU one level down, 2x2x2 stride-2 transposed conv back up, channel concat
    with the skip tensor, conv+ReLU.  Halos that cannot be recomputed locally arrive as face
    buffers (what the neighbour's halo_pack produced) and go in through halo_unpack.  Backward:
    activation-backward passes produce g tensors whose halos are exchanged the same way."""

    def __init__(self, x: Slab, params: dict, dout: torch.Tensor, faces: dict):
        from . import (ACT_RELU, FACE_D_HI, FACE_D_LO, POOL_MAX, act_bwd, concat_c, deconv2_bwd_data, deconv2_bwd_filter,
                       deconv2_fwd, halo_unpack, split_c)
        self.ws = Workspace()
        self.x, self.P, self.faces = x, params, faces
        dt, dev = x.t.dtype, x.t.device
        n, _, _, H, W = x.t.shape
        d, off, dg = x.d, x.d_offset, x.d_global
        ws, R, NONE = self.ws, ACT_RELU, ACT_NONE

        def slab(c, halo, level=1):
            s = 2 if level == 2 else 1
            t = torch.zeros((n, c, d // s + 2 * halo, H // s, W // s), dtype=dt, device=dev)
            return Slab(t, halo, halo, off // s, dg // s)

        def grads(name):
            w, b = params[name]
            return torch.empty(w.shape, dtype=torch.float32, device=dev), torch.empty(b.shape, dtype=torch.float32, device=dev)

        # The concatenation is not a copy: the skip tensor a2 and the up-sampled tensor ARE the two channel halves of
        # `cat` (views of its interior planes), written in place by the convolution and the transposed convolution that
        # produce them; in the backward pass the two halves of dcat are read in place the same way.
        T = self.T = {"a1": slab(32, 1), "p": slab(64, 2, 2), "b1": slab(64, 1, 2), "b2": slab(128, 0, 2),
                      "cat": slab(128, 1), "out": slab(64, 0)}
        T["a2"], T["up"] = T["cat"].channels(0, 64, 0, 0), T["cat"].channels(64, 128, 0, 0)
        G = self.G = {"dout": Slab(dout, 0, 0, off, dg), "g6": slab(64, 1), "dcat": slab(128, 0),
                      "d_b2": slab(128, 0, 2), "g4": slab(128, 1, 2), "d_b1": slab(64, 0, 2),
                      "g3": slab(64, 1, 2), "d_p": slab(64, 0, 2), "g2": slab(64, 1), "d_a1": slab(32, 0),
                      "g1": slab(32, 1), "dx": slab(1, 0)}
        G["d_skip"], G["d_up"] = G["dcat"].channels(0, 64), G["dcat"].channels(64, 128)
        self.dP = {k: grads(k) for k in params}
        self.ops = []

        es = x.t.element_size()

        def op(name, fn, flops=0, io=()):
            # algorithmic bytes of a call: every tensor it reads or writes once (stored planes, weights included)
            self.ops.append({"name": name, "fn": fn, "flops": int(flops), "bytes": int(sum(t.numel() * t.element_size() for t in io))})

        def cflops(name, out):   # 2*27*Cin*Cout per produced output voxel
            w = params[name][0]
            return 2 * 27 * w.shape[0] * w.shape[1] * out.t.numel() // out.t.shape[1]

        def exchange(name, t, width):
            lo, hi = faces[name]
            io = [f for f in (lo, hi) if f is not None] * 2
            op(f"halo_unpack_{name}", lambda: unpack_faces(lo, hi, t, width), 0, io)

        P = params
        W = {k: v[0] for k, v in params.items()}
        dflops = 2 * 128 * 64 * T["up"].t.numel() // 64
        op("c1_fwd", lambda: conv3d_fwd(x, *P["c1"], T["a1"], R, 0.0, ws), cflops("c1", T["a1"]), (x.t, T["a1"].t, W["c1"]))
        op("c2_fwd", lambda: conv3d_fwd(T["a1"], *P["c2"], T["a2"], R, 0.0, ws), cflops("c2", T["a2"]), (T["a1"].t, T["a2"].t, W["c2"]))
        op("pool_fwd", lambda: pool3d_fwd(T["a2"], T["p"], POOL_MAX), 0, (T["a2"].t, T["p"].interior))
        exchange("p", T["p"], 2)
        op("c3_fwd", lambda: conv3d_fwd(T["p"], *P["c3"], T["b1"], R, 0.0, ws), cflops("c3", T["b1"]), (T["p"].t, T["b1"].t, W["c3"]))
        op("c4_fwd", lambda: conv3d_fwd(T["b1"], *P["c4"], T["b2"], R, 0.0, ws), cflops("c4", T["b2"]), (T["b1"].t, T["b2"].t, W["c4"]))
        op("up_fwd", lambda: deconv2_fwd(T["b2"], *P["up"], T["up"], ws), dflops, (T["b2"].t, T["up"].t, W["up"]))
        exchange("cat", T["cat"], 1)
        op("c6_fwd", lambda: conv3d_fwd(T["cat"], *P["c6"], T["out"], R, 0.0, ws), cflops("c6", T["out"]), (T["cat"].t, T["out"].t, W["c6"]))
        self.n_fwd_ops = len(self.ops)
        # ---- backward
        dP = self.dP
        op("act_bwd_out", lambda: act_bwd(G["dout"], None, T["out"], G["g6"], R), 0, (G["dout"].t, T["out"].t, G["g6"].interior))
        exchange("g6", G["g6"], 1)
        op("c6_bwd_filter", lambda: conv3d_bwd_filter(T["cat"], G["g6"], None, *dP["c6"], NONE, 0.0, ws), cflops("c6", T["out"]),
           (T["cat"].t, G["g6"].interior, dP["c6"][0]))
        op("c6_bwd_data", lambda: conv3d_bwd_data(G["g6"], None, P["c6"][0], G["dcat"], NONE, 0.0, ws), cflops("c6", T["out"]),
           (G["g6"].t, G["dcat"].t, W["c6"]))
        op("up_bwd_filter", lambda: deconv2_bwd_filter(T["b2"], G["d_up"], *dP["up"], ws), dflops, (T["b2"].t, G["d_up"].t, dP["up"][0]))
        op("up_bwd_data", lambda: deconv2_bwd_data(G["d_up"], P["up"][0], G["d_b2"], ws), dflops, (G["d_up"].t, G["d_b2"].t, W["up"]))
        op("act_bwd_b2", lambda: act_bwd(G["d_b2"], None, T["b2"], G["g4"], R), 0, (G["d_b2"].t, T["b2"].t, G["g4"].interior))
        exchange("g4", G["g4"], 1)
        op("c4_bwd_filter", lambda: conv3d_bwd_filter(T["b1"], G["g4"], None, *dP["c4"], NONE, 0.0, ws), cflops("c4", T["b2"]),
           (T["b1"].t, G["g4"].interior, dP["c4"][0]))
        op("c4_bwd_data", lambda: conv3d_bwd_data(G["g4"], None, P["c4"][0], G["d_b1"], NONE, 0.0, ws), cflops("c4", T["b2"]),
           (G["g4"].t, G["d_b1"].t, W["c4"]))
        op("act_bwd_b1", lambda: act_bwd(G["d_b1"], None, T["b1"], G["g3"], R), 0, (G["d_b1"].t, T["b1"].interior, G["g3"].interior))
        exchange("g3", G["g3"], 1)
        op("c3_bwd_filter", lambda: conv3d_bwd_filter(T["p"], G["g3"], None, *dP["c3"], NONE, 0.0, ws), cflops("c3", G["d_b1"]),
           (T["p"].t, G["g3"].interior, dP["c3"][0]))
        op("c3_bwd_data", lambda: conv3d_bwd_data(G["g3"], None, P["c3"][0], G["d_p"], NONE, 0.0, ws), cflops("c3", G["d_b1"]),
           (G["g3"].t, G["d_p"].t, W["c3"]))
        # max-pooling backward, the skip branch's gradient and the activation derivative of a2 in one pass
        op("pool_bwd_act_a2", lambda: pool3d_bwd_act(G["d_p"], T["a2"], T["a2"], G["g2"], POOL_MAX, R, 0.0, G["d_skip"]), 0,
           (G["d_p"].t, T["a2"].t, G["d_skip"].t, G["g2"].interior))
        exchange("g2", G["g2"], 1)
        op("c2_bwd_filter", lambda: conv3d_bwd_filter(T["a1"], G["g2"], None, *dP["c2"], NONE, 0.0, ws), cflops("c2", T["a2"]),
           (T["a1"].t, G["g2"].interior, dP["c2"][0]))
        op("c2_bwd_data", lambda: conv3d_bwd_data(G["g2"], None, P["c2"][0], G["d_a1"], NONE, 0.0, ws), cflops("c2", T["a2"]),
           (G["g2"].t, G["d_a1"].t, W["c2"]))
        op("act_bwd_a1", lambda: act_bwd(G["d_a1"], None, T["a1"], G["g1"], R), 0, (G["d_a1"].t, T["a1"].interior, G["g1"].interior))
        exchange("g1", G["g1"], 1)
        op("c1_bwd_filter", lambda: conv3d_bwd_filter(x, G["g1"], None, *dP["c1"], NONE, 0.0, ws), cflops("c1", G["d_a1"]),
           (x.t, G["g1"].interior, dP["c1"][0]))
        op("c1_bwd_data", lambda: conv3d_bwd_data(G["g1"], None, P["c1"][0], G["dx"], NONE, 0.0, ws), cflops("c1", G["d_a1"]),
           (G["g1"].t, G["dx"].t, W["c1"]))

    def forward(self):
        for o in self.ops[:self.n_fwd_ops]:
            o["fn"]()

    def step(self):
        for o in self.ops:
            o["fn"]()

    def conv_flops(self) -> int:
        return sum(o["flops"] for o in self.ops)


class CosmoFlowShardChain:
    """The spatially-partitioned front of the Table I network on ONE depth shard (Sec. II-B, III-A): stages of
    3x3x3 convolution + leaky-ReLU + 2x2x2 average pooling whose inputs carry one halo plane per side.  Per stage,
    forward: halo_unpack of the two faces received from the depth neighbours, convolution (+ pooling; fused for the
    first stage), halo_pack of the pooled tensor's two faces for the neighbours; backward: pooling + activation
    backward into g, halo_pack / halo_unpack of g's faces, BF and BD.  The faces a neighbour would send are given
    as buffers (None at the global boundary: zero fill); the exchange itself is not part of this list.  After the
    last stage the paper redistributes the small tensor to sample parallelism; that stage's output has no halo."""

    def __init__(self, x: Slab, conv_params, dout: torch.Tensor, faces: dict, alpha: float = 0.01, fuse_pool: bool = True):
        from . import FACE_D_HI, FACE_D_LO, halo_bytes, halo_pack, halo_unpack
        self.ws = Workspace()
        ws, al = self.ws, alpha
        dt, dev = x.t.dtype, x.t.device
        es = x.t.element_size()
        n, L = x.t.shape[0], len(conv_params)
        self.conv = conv_params
        a, self.z, self.mask, self.g, self.da = [x], [], [], [], [None]
        for i, (w, _) in enumerate(conv_params):
            cur = a[i]
            H, W, co = cur.t.shape[3], cur.t.shape[4], w.shape[0]
            fused = bool(fuse_pool) and dt == torch.bfloat16 and w.shape[1] <= 4 and co <= 32 and cur.d % 2 == 0 and H % 2 == 0 and W % 16 == 0
            self.z.append(None if fused else Slab(torch.empty((n, co, cur.d, H, W), dtype=dt, device=dev), 0, 0, cur.d_offset, cur.d_global))
            self.mask.append(torch.empty((n * co * cur.d * H * W // 8,), dtype=torch.uint8, device=dev) if fused else None)
            self.g.append(Slab(torch.zeros((n, co, cur.d + 2, H, W), dtype=dt, device=dev), 1, 1, cur.d_offset, cur.d_global))
            halo = 1 if i < L - 1 else 0
            a.append(Slab(torch.zeros((n, co, cur.d // 2 + 2 * halo, H // 2, W // 2), dtype=dt, device=dev), halo, halo,
                          cur.d_offset // 2, cur.d_global // 2))
            self.da.append(Slab(dout, 0, 0, cur.d_offset // 2, cur.d_global // 2) if i == L - 1 else
                           Slab(torch.empty((n, co, cur.d // 2, H // 2, W // 2), dtype=dt, device=dev), 0, 0, cur.d_offset // 2, cur.d_global // 2))
        self.a = a
        self.da[0] = Slab(torch.empty((n, x.t.shape[1], x.d, x.t.shape[3], x.t.shape[4]), dtype=dt, device=dev), 0, 0, x.d_offset, x.d_global)
        self.dconv = [(torch.empty(w.shape, dtype=torch.float32, device=dev),
                       None if b is None else torch.empty(b.shape, dtype=torch.float32, device=dev)) for w, b in conv_params]
        send = lambda t: list(face_pair(t, 1))
        self.sent = {}
        self.ops = []

        def op(name, fn, flops=0, nbytes=0):
            self.ops.append({"name": name, "fn": fn, "flops": int(flops), "bytes": int(nbytes)})

        def unpack(name, t):
            lo, hi = faces[name]
            op(f"halo_unpack_{name}", lambda: unpack_faces(lo, hi, t, 1), 0, 4 * halo_bytes(t, 1))

        def pack(name, t):
            bufs = self.sent[name] = send(t)
            op(f"halo_pack_{name}", lambda: pack_faces(t, 1, bufs[0], bufs[1]), 0, 4 * halo_bytes(t, 1))

        for i, (w, b) in enumerate(conv_params):
            cur, nxt, z, mask, g = a[i], a[i + 1], self.z[i], self.mask[i], self.g[i]
            vox = n * cur.d * cur.t.shape[3] * cur.t.shape[4]
            fl = 2 * 27 * w.shape[1] * w.shape[0] * vox
            unpack(f"a{i}", cur)
            if z is None:
                zshape = (n, w.shape[0], cur.d, cur.t.shape[3], cur.t.shape[4])
                op(f"conv{i + 1}_fwd_pool", lambda cur=cur, w=w, b=b, zshape=zshape, nxt=nxt, mask=mask: conv3d_fwd_pool(
                    cur, w, b, zshape, nxt, mask, ACT_LEAKY, al, ws), fl, (cur.t.numel() + vox * w.shape[0] // 8) * es + mask.numel())
            else:
                op(f"conv{i + 1}_fwd", lambda cur=cur, w=w, b=b, z=z: conv3d_fwd(cur, w, b, z, ACT_LEAKY, al, ws), fl,
                   (cur.t.numel() + z.t.numel()) * es)
                op(f"pool{i + 1}_fwd", lambda z=z, nxt=nxt: pool3d_fwd(z, nxt, POOL_AVG), 0, z.t.numel() * es * 9 // 8)
            if i < L - 1:
                pack(f"a{i + 1}", nxt)
        self.n_fwd_ops = len(self.ops)
        for i in range(L - 1, -1, -1):
            w = conv_params[i][0]
            cur, z, mask, g, dp = a[i], self.z[i], self.mask[i], self.g[i], self.da[i + 1]
            vox = n * cur.d * cur.t.shape[3] * cur.t.shape[4]
            fl = 2 * 27 * w.shape[1] * w.shape[0] * vox
            if z is None:
                op(f"pool{i + 1}_bwd_mask", lambda dp=dp, mask=mask, g=g: pool3d_bwd_mask(dp, mask, g, ACT_LEAKY, al), 0,
                   (dp.t.numel() + vox * w.shape[0]) * es + mask.numel())
            else:
                op(f"pool{i + 1}_bwd_act", lambda dp=dp, z=z, g=g: pool3d_bwd_act(dp, None, z, g, POOL_AVG, ACT_LEAKY, al), 0,
                   (dp.t.numel() + 2 * z.t.numel()) * es)
            pack(f"g{i + 1}", g)
            unpack(f"g{i + 1}", g)
            op(f"conv{i + 1}_bwd_filter", lambda cur=cur, g=g, i=i: conv3d_bwd_filter(cur, g, None, self.dconv[i][0], self.dconv[i][1],
                                                                                       ACT_NONE, 0.0, ws), fl, (cur.t.numel() + vox * w.shape[0]) * es)
            op(f"conv{i + 1}_bwd_data", lambda g=g, w=w, i=i: conv3d_bwd_data(g, None, w, self.da[i], ACT_NONE, 0.0, ws), fl,
               (g.t.numel() + self.da[i].t.numel()) * es)

    def forward(self):
        for o in self.ops[:self.n_fwd_ops]:
            o["fn"]()

    def step(self):
        for o in self.ops:
            o["fn"]()

    def conv_flops(self) -> int:
        return sum(o["flops"] for o in self.ops)


class SingleLayer:
    """One conv3d layer on a depth shard with its pooling and halo traffic, as a list of calls:
    halo_unpack of both D faces, conv fwd (+bias+act), pool fwd, halo_pack of the input faces;
    pool bwd fused with the activation backward, BF and BD on g (g carries a 1-plane halo).
    The caller brings the tensors that hold values (x with its halo planes, w, b, the gradient slab g with a halo
    plane per side, the pooled gradient dp when pooling is on); buffers that are only written are made here."""

    def __init__(self, x: Slab, w, b, g: Slab, dp: Slab | None = None, pool=True, act=ACT_LEAKY, alpha=0.01, split=False, faces_hw=False,
                 fuse_pool=False, halo_ops=True):
        from . import FACE_D_HI, FACE_D_LO, halo_bytes, halo_pack, halo_unpack
        dev, dtype = x.t.device, x.t.dtype
        n, cin, _, hw, _ = x.t.shape
        cout, d, d_offset, d_global = w.shape[0], x.d, x.d_offset, x.d_global
        self.ws = Workspace()
        ws, es = self.ws, x.t.element_size()
        self.x, self.w, self.b, self.g = x, w, b, g
        # fuse_pool: convolution, activation and average pooling in one call; the unpooled activation is not stored, a
        # sign mask (one bit per voxel) stands in for it in the pooling backward (first-layer shapes, bf16)
        fused = self.fused = bool(fuse_pool and pool and not split and dtype == torch.bfloat16 and cin <= 4 and cout <= 32
                                  and d % 2 == 0 and hw % 16 == 0)
        z = self.z = None if fused else Slab(torch.empty((n, cout, d, hw, hw), dtype=dtype, device=dev), 0, 0, d_offset, d_global)
        dx = self.dx = Slab(torch.empty((n, cin, d, hw, hw), dtype=dtype, device=dev), 0, 0, d_offset, d_global)
        self.dw = torch.empty((cout, cin, 3, 3, 3), device=dev)
        self.db = torch.empty((cout,), device=dev)
        faces, gfaces = face_pair(x, 1), face_pair(g, 1)      # (what goes out to the neighbours comes back in: a stand-in for theirs)
        self.ops = []
        fl = 2 * 27 * cin * cout * n * d * hw * hw
        vox = n * d * hw * hw

        def op(name, fn, flops=0, nbytes=0):
            self.ops.append({"name": name, "fn": fn, "flops": int(flops), "bytes": int(nbytes)})

        # halo_ops=False: an unsharded volume (d_offset 0, d_global = d) has no neighbours and no face traffic
        if halo_ops:
            op("halo_pack_x", lambda: pack_faces(x, 1, faces[0], faces[1]), 0, 4 * faces[0].numel() * es)
            op("halo_unpack_x", lambda: unpack_faces(faces[0], faces[1], x, 1), 0, 4 * faces[0].numel() * es)
        if fused:
            p = self.p = Slab(torch.empty((n, cout, d // 2, hw // 2, hw // 2), dtype=dtype, device=dev), 0, 0, d_offset // 2, d_global // 2)
            mask = self.mask = torch.empty((n * cout * d * hw * hw // 8,), dtype=torch.uint8, device=dev)
            op("conv_fwd_pool", lambda: conv3d_fwd_pool(x, w, b, (n, cout, d, hw, hw), p, mask, act, alpha, ws), fl,
               (x.t.numel() + p.t.numel() + w.numel()) * es + mask.numel())
        else:
            op("conv_fwd", lambda: conv3d_fwd(x, w, b, z, act, alpha, ws), fl, (x.t.numel() + z.t.numel() + w.numel()) * es)
        if split and d >= 3:
            # the same forward as main planes (no halo needed) + the two one-plane strips (Sec. III-C), on plane-run views
            pl = n * hw * hw
            op("conv_fwd_main", lambda: conv3d_fwd(x.planes(1, d - 1, 1, 1), w, b, z.planes(1, d - 1), act, alpha, ws),
               fl * (d - 2) // d, (pl * (d * cin + (d - 2) * cout) + w.numel()) * es)
            op("conv_fwd_strips", lambda: (conv3d_fwd(x.planes(0, 1, 1, 1), w, b, z.planes(0, 1), act, alpha, ws),
                                           conv3d_fwd(x.planes(d - 1, d, 1, 1), w, b, z.planes(d - 1, d), act, alpha, ws)),
               fl * 2 // d, (pl * 2 * (3 * cin + cout) + 2 * w.numel()) * es)
        if pool and fused:
            self.dp = dp
            op("pool_bwd_mask", lambda: pool3d_bwd_mask(dp, mask, g, act, alpha), 0, (dp.t.numel() + vox * cout) * es + mask.numel())
        elif pool:
            p = self.p = Slab(torch.empty((n, cout, d // 2, hw // 2, hw // 2), dtype=dtype, device=dev), 0, 0, d_offset // 2, d_global // 2)
            self.dp = dp
            op("pool_fwd", lambda: pool3d_fwd(z, p, POOL_AVG), 0, (z.t.numel() + p.t.numel()) * es)
            op("pool_bwd_act", lambda: pool3d_bwd_act(dp, None, z, g, POOL_AVG, act, alpha), 0, (dp.t.numel() + 2 * z.t.numel()) * es)
        if halo_ops:
            op("halo_pack_g", lambda: pack_faces(g, 1, gfaces[0], gfaces[1]), 0, 4 * gfaces[0].numel() * es)
            op("halo_unpack_g", lambda: unpack_faces(gfaces[0], gfaces[1], g, 1), 0, 4 * gfaces[0].numel() * es)
        if faces_hw:
            # H and W faces of the activation gradient (a partitioning in H or W as well, Sec. II-B): one and two
            # voxels wide, pack and unpack of both ends; bytes = face read + face written
            from . import box_pack, box_unpack
            ds, H, W = g.t.shape[2], g.t.shape[3], g.t.shape[4]
            for wd_ in (1, 2):
                hb = [torch.empty((n, cout, ds, wd_, W), dtype=dtype, device=dev) for _ in range(2)]
                wb = [torch.empty((n, cout, ds, H, wd_), dtype=dtype, device=dev) for _ in range(2)]
                op(f"face_pack_h{wd_}", lambda hb=hb, k=wd_: (box_pack(g.t, (0, 0, 0, ds, k, W), hb[0]), box_pack(g.t, (0, H - k, 0, ds, k, W), hb[1])),
                   0, 4 * hb[0].numel() * es)
                op(f"face_unpack_h{wd_}", lambda hb=hb, k=wd_: (box_unpack(hb[1], g.t, (0, 0, 0, ds, k, W)), box_unpack(hb[0], g.t, (0, H - k, 0, ds, k, W))),
                   0, 4 * hb[0].numel() * es)
                op(f"face_pack_w{wd_}", lambda wb=wb, k=wd_: (box_pack(g.t, (0, 0, 0, ds, H, k), wb[0]), box_pack(g.t, (0, 0, W - k, ds, H, k), wb[1])),
                   0, 4 * wb[0].numel() * es)
                op(f"face_unpack_w{wd_}", lambda wb=wb, k=wd_: (box_unpack(wb[1], g.t, (0, 0, 0, ds, H, k)), box_unpack(wb[0], g.t, (0, 0, W - k, ds, H, k))),
                   0, 4 * wb[0].numel() * es)
        op("conv_bwd_filter", lambda: conv3d_bwd_filter(x, g, None, self.dw, self.db, ACT_NONE, 0.0, ws), fl,
           (x.t.numel() + vox * cout) * es + w.numel() * 4)
        op("conv_bwd_data", lambda: conv3d_bwd_data(g, None, w, dx, ACT_NONE, 0.0, ws), fl, (g.t.numel() + dx.t.numel() + w.numel()) * es)

    def step(self):
        for o in self.ops:
            o["fn"]()

    def conv_flops(self):
        return sum(o["flops"] for o in self.ops)


class BatchNormLayer:
    """The local passes of one distributed batch-normalisation layer on a slab, as a list of calls (the allreduce of
    the per-channel sums between them is the caller's and is not part of this list).  x, dy: the caller's tensors."""

    def __init__(self, x: Slab, dy: Slab):
        from . import bn_bwd, bn_bwd_stats, bn_finalize, bn_fwd, bn_stats
        dev = x.t.device
        n, c, _, hw, _ = x.t.shape
        d = x.d
        self.ws = Workspace()
        ws, es = self.ws, x.t.element_size()
        y, dx = Slab(torch.empty_like(x.t)), Slab(torch.empty_like(x.t))
        vec = lambda: torch.empty(c, device=dev)
        s, sq, mean, invstd, sdy, sdx = vec(), vec(), vec(), vec(), vec(), vec()
        gamma, beta = torch.ones(c, device=dev), torch.zeros(c, device=dev)
        count, nb = n * d * hw * hw, x.t.numel() * es
        self.keep = (x, dy, y, dx)
        self.ops = []

        def op(name, fn, nbytes):
            self.ops.append({"name": name, "fn": fn, "flops": 0, "bytes": int(nbytes)})

        op("bn_stats", lambda: bn_stats(x, s, sq, ws), nb)
        op("bn_finalize", lambda: bn_finalize(s, sq, count, 1e-5, mean, invstd), 0)
        op("bn_fwd", lambda: bn_fwd(x, mean, invstd, gamma, beta, y, ws), 2 * nb)
        op("bn_bwd_stats", lambda: bn_bwd_stats(dy, x, mean, invstd, sdy, sdx, ws), 2 * nb)
        op("bn_bwd", lambda: bn_bwd(dy, x, mean, invstd, gamma, sdy, sdx, count, dx, ws), 3 * nb)

    def step(self):
        for o in self.ops:
            o["fn"]()

    def conv_flops(self):
        return 0
