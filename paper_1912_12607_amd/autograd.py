"""PyTorch autograd plug-in over the C ABI: an INT8 convolution layer whose forward, backward-data
and backward-weight passes run on int8 codes (Sec.3.1 Eq.1-3, Sec.3.4), with the gradient clip
chosen by the Direction Sensitive Gradient Clipping search and the layer's deviation d_c exposed for
Deviation Counteractive LR Scaling (Sec.3.5 Eq.7).

Plumbing only: every arithmetic step is one of the library's entry points; torch supplies device
memory, the stream and the autograd graph.  CUDA(ROCm) tensors, fp32, contiguous NCHW.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from .inputs import default_ratios


def _scratch(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(256, nbytes), dtype=torch.uint8, device=device)


class _Int8ConvFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, w, layer):
        x = x.contiguous()
        w = w.contiguous()
        N, C, H, W = x.shape
        K, Cg, R, S = w.shape
        dev = x.device
        desc = B.make_desc(N, C, H, W, K, R, S, layer.stride, layer.padding, layer.groups)
        depthwise = layer.groups != 1
        act_kind = B.ACT_PLANAR if depthwise else B.ACT
        wgt_kind = B.WGT_PLANAR if depthwise else B.WGT
        P = (H + 2 * layer.padding[0] - R) // layer.stride[0] + 1
        Q = (W + 2 * layer.padding[1] - S) // layer.stride[1] + 1
        i8, f32 = torch.int8, torch.float32
        xq = torch.empty(B.int8t_code_bytes(x.shape, act_kind), dtype=i8, device=dev)
        wq = torch.empty(B.int8t_code_bytes(w.shape, wgt_kind), dtype=i8, device=dev)
        sx = torch.empty(1, dtype=f32, device=dev)
        sw = torch.empty(1, dtype=f32, device=dev)
        # activations and weights in one batched call (one absmax launch, one quantize launch)
        items = [(x, tuple(x.shape), act_kind, None, xq, sx), (w, tuple(w.shape), wgt_kind, None, wq, sw)]
        B.int8t_quantize_batch(items, _scratch(B.int8t_quantize_batch_workspace_bytes(items), dev))
        y = torch.empty((N, K, P, Q), dtype=f32, device=dev)
        nf = B.int8t_workspace_bytes(B.OP_CONV_FWD, desc)
        B.int8t_conv_fwd(desc, xq, sx, wq, sw, y, None, _scratch(nf, dev) if nf else None)
        ctx.layer, ctx.desc, ctx.act_kind = layer, desc, act_kind
        ctx.x_shape, ctx.w_shape = tuple(x.shape), tuple(w.shape)
        ctx.save_for_backward(xq, sx, wq, sw)
        return y

    @staticmethod
    def backward(ctx, dy):
        xq, sx, wq, sw = ctx.saved_tensors
        layer, desc = ctx.layer, ctx.desc
        dy = dy.contiguous()
        dev = dy.device
        i8, f32, f64 = torch.int8, torch.float32, torch.float64
        n_y = dy.numel()
        seed = layer.next_seed()
        ws = _scratch(max(B.int8t_workspace_bytes(B.OP_DSGC, None, n_y, layer.ratios.numel()),
                          B.int8t_quantize_workspace_bytes(dy.shape, ctx.act_kind),
                          B.int8t_workspace_bytes(B.OP_CONV_BWD_WEIGHT, desc),
                          B.int8t_workspace_bytes(B.OP_CONV_BWD_DATA, desc)), dev)
        if layer.clip is None:
            layer.clip = torch.empty(1, dtype=f32, device=dev)
            layer.deviation = torch.zeros(1, dtype=f64, device=dev)
        # Periodic Update (Sec.3.4): the clip value is searched every `dsgc_period` backward passes
        if layer.backward_calls % layer.dsgc_period == 0:
            B.int8t_dsgc_clip(dy, n_y, layer.ratios, layer.ratios.numel(), B.ROUND_STOCHASTIC, seed,
                              layer.clip, layer.deviation, None, ws)
            dev_out = None
        else:
            dev_out = layer.deviation          # Eq.6 of the codes actually produced with the kept clip
        layer.backward_calls += 1
        dyq = torch.empty(B.int8t_code_bytes(dy.shape, ctx.act_kind), dtype=i8, device=dev)
        sdy = torch.empty(1, dtype=f32, device=dev)
        B.int8t_quantize(dy, dy.shape, ctx.act_kind, layer.clip, B.ROUND_STOCHASTIC, seed, dyq, sdy, dev_out, ws)
        dx = dw = None
        if ctx.needs_input_grad[0]:
            dx = torch.empty(ctx.x_shape, dtype=f32, device=dev)
            B.int8t_conv_bwd_data(desc, dyq, sdy, wq, sw, dx, None, ws)
        if ctx.needs_input_grad[1]:
            dw = torch.empty(ctx.w_shape, dtype=f32, device=dev)
            B.int8t_conv_bwd_weight(desc, xq, sx, dyq, sdy, dw, None, ws)
        return dx, dw, None


class Int8Conv2d(torch.nn.Module):
    """Drop-in for a bias-free `torch.nn.Conv2d` (groups 1 or depthwise).  After a backward pass
    `deviation` holds d_c of this layer's output gradient (device, fp64) and `dclr_scale()` the
    factor phi(d_c) of Eq.7 to multiply this layer's learning rate with."""

    def __init__(self, in_channels, out_channels, kernel_size, stride=1, padding=0, groups=1,
                 n_candidates: int = 32, dsgc_period: int = 1, seed: int = 0, device="cuda:0"):
        super().__init__()
        pair = lambda v: (v, v) if isinstance(v, int) else tuple(v)
        self.kernel_size, self.stride, self.padding, self.groups = pair(kernel_size), pair(stride), pair(padding), groups
        assert groups == 1 or (groups == in_channels == out_channels), "groups 1 or depthwise"
        fan_in = (in_channels // groups) * self.kernel_size[0] * self.kernel_size[1]
        w = torch.randn(out_channels, in_channels // groups, *self.kernel_size, device=device) * (2.0 / fan_in) ** 0.5
        self.weight = torch.nn.Parameter(w)
        self.ratios = torch.from_numpy(np.ascontiguousarray(default_ratios(n_candidates))).to(device)
        self.dsgc_period = max(1, int(dsgc_period))
        self.backward_calls = 0
        self.clip = None
        self.deviation = None
        self._seed = int(seed)

    def next_seed(self) -> int:
        self._seed += 1
        return self._seed

    def forward(self, x):
        return _Int8ConvFn.apply(x, self.weight, self)

    def dclr_scale(self, alpha: float = 20.0, beta: float = 0.1) -> float:
        """phi(d_c) = max(exp(-alpha d_c), beta) for the last backward pass (reads d_c back)."""
        if self.deviation is None:
            return 1.0
        return B.int8t_dclr_scale(float(self.deviation.item()), alpha, beta)


class DclrSGD(torch.optim.SGD):
    """SGD whose learning rate is scaled per INT8 layer by phi(d_c) of that layer's last backward
    pass: Deviation Counteractive LR Scaling, Sec.3.5 Eq.7.  Parameters that belong to no
    `Int8Conv2d` keep the base rate.  `step()` reads each layer's d_c back from the device."""

    def __init__(self, model: torch.nn.Module, lr: float, alpha: float = 20.0, beta: float = 0.1, **sgd_kwargs):
        self.alpha, self.beta = alpha, beta
        self._layers = [m for m in model.modules() if isinstance(m, Int8Conv2d)]
        int8_ids = {id(m.weight) for m in self._layers}
        rest = [p for p in model.parameters() if id(p) not in int8_ids]
        groups = [{"params": [m.weight], "base_lr": lr} for m in self._layers]
        if rest:
            groups.append({"params": rest, "base_lr": lr})
        super().__init__(groups, lr=lr, **sgd_kwargs)

    def set_lr(self, lr: float):
        """New base rate (schedulers act on this, the DCLR factor is applied on top)."""
        for g in self.param_groups:
            g["base_lr"] = lr

    @torch.no_grad()
    def step(self, closure=None):
        for g, m in zip(self.param_groups, self._layers):
            g["lr"] = g["base_lr"] * m.dclr_scale(self.alpha, self.beta)
        for g in self.param_groups[len(self._layers):]:
            g["lr"] = g["base_lr"]
        return super().step(closure)

