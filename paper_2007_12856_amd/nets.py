"""Call sequences of the two network shapes over the C-ABI binding (no arithmetic here: every
step is one library call; buffers are allocated once, a step allocates nothing).

CosmoFlowStack: conv3d 3x3x3 + leaky-ReLU + 2x2x2 average pooling stages, flatten, three
fully-connected layers, MSE loss (the network of Table I, Sec. IV, in the 5-stage shape the
benchmark configuration names), forward and backward (BD and BF of every layer, Sec. III-C).
"""
from __future__ import annotations

import torch

from . import (ACT_LEAKY, ACT_NONE, POOL_AVG, Slab, Workspace, conv3d_bwd_data, conv3d_bwd_filter, conv3d_fwd,
               dense_bwd, dense_fwd, mse_fwd_bwd, pool3d_bwd, pool3d_fwd)


class CosmoFlowStack:
    def __init__(self, x: torch.Tensor, target: torch.Tensor, conv_params, fc_params, alpha: float = 0.01):
        """x [N,C,D,H,W] device tensor; conv_params/fc_params: lists of (w, bias) device tensors
        (w in x's dtype, bias fp32); target fp32 [N, nout]."""
        self.alpha = alpha
        self.ws = Workspace()
        dt, dev = x.dtype, x.device
        self.x = Slab(x)
        self.target = target
        self.conv, self.fc = conv_params, fc_params
        n = x.shape[0]
        self.z, self.p = [], []
        cur = self.x
        for w, _ in conv_params:
            z = cur.like(w.shape[0])
            p = Slab(torch.empty((n, w.shape[0], cur.d // 2, cur.t.shape[3] // 2, cur.t.shape[4] // 2), dtype=dt, device=dev))
            self.z.append(z)
            self.p.append(p)
            cur = p
        self.flat = cur.t.view(n, -1)
        self.y = [torch.empty((n, w.shape[0]), dtype=dt, device=dev) for w, _ in fc_params]
        self.loss = torch.empty((1,), dtype=torch.float32, device=dev)
        # gradients
        self.dy = [torch.empty_like(y) for y in self.y]
        self.dfc = [(torch.empty(w.shape, dtype=torch.float32, device=dev), torch.empty(b.shape, dtype=torch.float32, device=dev))
                    for w, b in fc_params]
        self.dp = [Slab(torch.empty_like(p.t)) for p in self.p]
        self.dz = [Slab(torch.empty_like(z.t)) for z in self.z]
        self.dx = Slab(torch.empty_like(x))
        self.dconv = [(torch.empty(w.shape, dtype=torch.float32, device=dev), torch.empty(b.shape, dtype=torch.float32, device=dev))
                      for w, b in conv_params]

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
            fl = 2 * 27 * w.shape[1] * w.shape[0] * z.t.numel() // w.shape[0]
            io = (cur.t.numel() + z.t.numel() + w.numel()) * es
            self._op(f"conv{i + 1}_fwd", lambda cur=cur, w=w, b=b, z=z: conv3d_fwd(cur, w, b, z, ACT_LEAKY, al, ws), fl, io)
            self._op(f"pool{i + 1}_fwd", lambda z=z, p=p: pool3d_fwd(z, p, POOL_AVG), 0, (z.t.numel() + p.t.numel()) * es)
            cur = p
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
            dxin = self.dp[-1].t.view(xin.shape) if i == 0 else self.dy[i - 1]
            w = self.fc[i][0]
            act = ACT_NONE if i == last else ACT_LEAKY
            self._op(f"fc{i + 1}_bwd", lambda xin=xin, w=w, i=i, dxin=dxin, act=act: dense_bwd(
                xin, w, self.y[i], self.dy[i], dxin, self.dfc[i][0], self.dfc[i][1], act, al),
                4 * xin.shape[0] * w.numel(), w.numel() * es + w.numel() * 4)
        for i in range(nconv - 1, -1, -1):
            w = self.conv[i][0]
            z, dz, dp = self.z[i], self.dz[i], self.dp[i]
            xin = self.x if i == 0 else self.p[i - 1]
            dxin = self.dx if i == 0 else self.dp[i - 1]
            fl = 2 * 27 * w.shape[1] * w.shape[0] * z.t.numel() // w.shape[0]
            self._op(f"pool{i + 1}_bwd", lambda dp=dp, dz=dz: pool3d_bwd(dp, None, dz, POOL_AVG), 0, (dp.t.numel() + dz.t.numel()) * es)
            self._op(f"conv{i + 1}_bwd_filter", lambda xin=xin, dz=dz, z=z, i=i: conv3d_bwd_filter(
                xin, dz, z, self.dconv[i][0], self.dconv[i][1], ACT_LEAKY, al, ws), fl,
                (xin.t.numel() + dz.t.numel() + z.t.numel()) * es + w.numel() * 4)
            self._op(f"conv{i + 1}_bwd_data", lambda dz=dz, z=z, w=w, dxin=dxin: conv3d_bwd_data(dz, z, w, dxin, ACT_LEAKY, al, ws),
                     fl, (dz.t.numel() + z.t.numel() + dxin.t.numel() + w.numel()) * es)

    def forward(self):
        for op in self.ops[:self.n_fwd_ops]:
            op["fn"]()
        return self.y[-1]

    def backward(self):
        for op in self.ops[self.n_fwd_ops:]:
            op["fn"]()

    def step(self):
        for op in self.ops:
            op["fn"]()

    def conv_flops(self) -> int:
        return sum(op["flops"] for op in self.ops if op["name"].startswith("conv"))
