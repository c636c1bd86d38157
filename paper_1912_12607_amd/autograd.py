"""PyTorch autograd plug-in over the C ABI: INT8 convolution and fully connected layers whose forward,
backward-data and backward-weight passes run on int8 codes (Sec.3.1 Eq.1-3, Sec.3.4), with the
gradient clip chosen by the Direction Sensitive Gradient Clipping search, the layer's deviation d_c
exposed for Deviation Counteractive LR Scaling (Sec.3.5 Eq.7), and `replace_modules()`, the
"automatic match and replacement" of a model's convolution and fully connected layers by their 8-bit
counterparts (Sec.3.6 item 1).

Plumbing only: every arithmetic step of the INT8 path is one of the library's entry points; torch
supplies device memory, the stream and the autograd graph (and adds the fp32 bias, which like the
normalisation layers stays unquantized, Sec.4).  CUDA(ROCm) tensors, fp32, contiguous NCHW.
"""
from __future__ import annotations

import zlib

import numpy as np
import torch

from . import binding as B
from .inputs import default_ratios


class _LayerBuffers:
    """Device buffers of one layer at one input shape, allocated once and kept: scratch, the codes of
    the weights and of the output gradient, the scalars.  The codes of the activations are the one
    thing a forward pass must keep until its backward pass: they come from a small pool per shape
    (taken in forward, handed back in backward), so a layer called several times before its backward
    passes keeps each call's codes apart, and a steady training loop allocates nothing."""

    def __init__(self, layer, x_shape, dev):
        N, C, H, W = x_shape
        K, Cg, R, S = layer.weight_shape
        self.desc = B.make_desc(N, C, H, W, K, R, S, layer.stride, layer.padding, layer.groups)
        depthwise = layer.groups != 1
        self.act_kind = B.ACT_PLANAR if depthwise else B.ACT
        self.wgt_kind = B.WGT_PLANAR if depthwise else B.WGT
        P = (H + 2 * layer.padding[0] - R) // layer.stride[0] + 1
        Q = (W + 2 * layer.padding[1] - S) // layer.stride[1] + 1
        self.x_shape, self.w_shape, self.y_shape = (N, C, H, W), (K, Cg, R, S), (N, K, P, Q)
        i8, f32, u8 = torch.int8, torch.float32, torch.uint8
        self.dev = dev
        self.wq = torch.empty(B.int8t_code_bytes(self.w_shape, self.wgt_kind), dtype=i8, device=dev)
        self.dyq = torch.empty(B.int8t_code_bytes(self.y_shape, self.act_kind), dtype=i8, device=dev)
        self.sw = torch.empty(1, dtype=f32, device=dev)
        self.sdy = torch.empty(1, dtype=f32, device=dev)
        self.xq_bytes = B.int8t_code_bytes(self.x_shape, self.act_kind)
        self.xq_pool = []
        n_y = N * K * P * Q
        nq = B.int8t_quantize_batch_workspace_bytes(
            [(None, self.x_shape, self.act_kind, None, None, None), (None, self.w_shape, self.wgt_kind, None, None, None)])
        nbytes = max(256, nq, B.int8t_workspace_bytes(B.OP_CONV_FWD, self.desc),
                     B.int8t_workspace_bytes(B.OP_DSGC, None, n_y, layer.ratios.numel()),
                     B.int8t_quantize_workspace_bytes(self.y_shape, self.act_kind),
                     B.int8t_workspace_bytes(B.OP_CONV_BWD_WEIGHT, self.desc),
                     B.int8t_workspace_bytes(B.OP_CONV_BWD_DATA, self.desc))
        self.ws = torch.empty(nbytes, dtype=u8, device=dev)

    def take_xq(self):
        if self.xq_pool:
            return self.xq_pool.pop()
        return (torch.empty(self.xq_bytes, dtype=torch.int8, device=self.dev),
                torch.empty(1, dtype=torch.float32, device=self.dev))

    def give_xq(self, pair):
        self.xq_pool.append(pair)


class _Int8ConvFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, w, layer, keep):
        x = x.contiguous()
        w = w.contiguous()
        buf = layer.buffers(tuple(x.shape), x.device)
        xq, sx = buf.take_xq()
        # activations and weights in one batched call (one absmax launch, one quantize launch)
        B.int8t_quantize_batch([(x, buf.x_shape, buf.act_kind, None, xq, sx), (w, buf.w_shape, buf.wgt_kind, None, buf.wq, buf.sw)],
                               buf.ws)
        y = torch.empty(buf.y_shape, dtype=torch.float32, device=x.device)
        B.int8t_conv_fwd(buf.desc, xq, sx, buf.wq, buf.sw, y, None, buf.ws)
        if keep:      # a backward pass will come for the codes
            ctx.layer, ctx.buf, ctx.xq = layer, buf, (xq, sx)
            ctx.w_version = layer.weight._version
        else:
            buf.give_xq((xq, sx))
        return y

    @staticmethod
    def backward(ctx, dy):
        layer, buf = ctx.layer, ctx.buf
        xq, sx = ctx.xq
        dy = dy.contiguous()
        n_y = dy.numel()
        seed = layer.next_seed()
        if layer.clip is None:
            layer.clip = torch.empty(1, dtype=torch.float32, device=dy.device)
            layer.deviation = torch.zeros(1, dtype=torch.float64, device=dy.device)
        # Periodic Update (Sec.3.4): the clip value is searched every `dsgc_period` backward passes
        if layer.backward_calls % layer.dsgc_period == 0:
            J = layer.ratios.numel()
            refine = layer.dsgc_refine
            B.int8t_dsgc_clip(dy, n_y, layer.ratios, J, B.ROUND_STOCHASTIC, seed,
                              layer.clip, layer.deviation, layer.dev_all if refine else None, buf.ws)
            # Refinement of the clip value (Sec.3.4 learns c by descending d_c; no step size is given): further
            # sweeps over J candidates spaced geometrically around the last winner, the window shrinking by the
            # factor J / 2 each time.  The winner itself is candidate J / 2, so d_c never rises.  The ratios are
            # formed on the device (no host round trip): winner's ratio times 2^((j - J/2) * w / J), capped at 1.
            ratios, width = layer.ratios, layer.ratio_step
            for _ in range(refine):
                best = torch.argmin(layer.dev_all[:J])
                ratios = torch.clamp(ratios[best] * layer.refine_factors(width), max=1.0)
                B.int8t_dsgc_clip(dy, n_y, ratios, J, B.ROUND_STOCHASTIC, seed,
                                  layer.clip, layer.deviation, layer.dev_all, buf.ws)
                width = 2.0 * width / J
            layer.last_ratios = ratios          # the candidates of the last sweep (the grid itself without refinement)
            dev_out = None
        else:
            dev_out = layer.deviation          # Eq.6 of the codes actually produced with the kept clip
        layer.backward_calls += 1
        B.int8t_quantize(dy, buf.y_shape, buf.act_kind, layer.clip, B.ROUND_STOCHASTIC, seed, buf.dyq, buf.sdy, dev_out, buf.ws)
        if layer.weight._version != ctx.w_version:
            # the weights changed between this layer's forward and backward pass (an optimizer step in
            # between): the codes of W the forward used are gone, quantize the current ones again
            B.int8t_quantize(layer.weight.detach().contiguous().view(buf.w_shape), buf.w_shape, buf.wgt_kind, None, B.ROUND_NEAREST_EVEN, 0,
                             buf.wq, buf.sw, None, buf.ws)
        dx = dw = None
        if ctx.needs_input_grad[0]:
            dx = torch.empty(buf.x_shape, dtype=torch.float32, device=dy.device)
            B.int8t_conv_bwd_data(buf.desc, buf.dyq, buf.sdy, buf.wq, buf.sw, dx, None, buf.ws)
        if ctx.needs_input_grad[1]:
            dw = torch.empty(buf.w_shape, dtype=torch.float32, device=dy.device)
            B.int8t_conv_bwd_weight(buf.desc, xq, sx, buf.dyq, buf.sdy, dw, None, buf.ws)
        buf.give_xq((xq, sx))
        ctx.xq = None
        return dx, dw, None, None


def _pair(v):
    return (v, v) if isinstance(v, int) else tuple(v)


class Int8Conv2d(torch.nn.Module):
    """Drop-in for `torch.nn.Conv2d` (groups 1 or depthwise, dilation 1, zero padding).  The bias, if
    any, stays fp32 and is added to the dequantized result.  After a backward pass `deviation` holds
    d_c of this layer's output gradient (device, fp64) and `dclr_scale()` the factor phi(d_c) of Eq.7
    to multiply this layer's learning rate with."""

    def __init__(self, in_channels, out_channels, kernel_size, stride=1, padding=0, groups=1, bias=False,
                 n_candidates: int = 32, dsgc_period: int = 1, dsgc_refine: int = 0, seed: int | None = None,
                 device="cuda:0", name: str = ""):
        """dsgc_refine: sweeps that refine the clip value around the winner of the candidate grid (0: the grid only)."""
        super().__init__()
        self.in_channels, self.out_channels = in_channels, out_channels
        self.kernel_size, self.stride, self.padding, self.groups = _pair(kernel_size), _pair(stride), _pair(padding), groups
        assert groups == 1 or (groups == in_channels == out_channels), "groups 1 or depthwise"
        fan_in = (in_channels // groups) * self.kernel_size[0] * self.kernel_size[1]
        w = torch.randn(out_channels, in_channels // groups, *self.kernel_size, device=device) * (2.0 / fan_in) ** 0.5
        self.weight = torch.nn.Parameter(w)
        self.weight_shape = tuple(w.shape)      # K, C/groups, R, S (the Parameter of Int8Linear is K, C)
        self.bias = torch.nn.Parameter(torch.zeros(out_channels, device=device)) if bias else None
        self.ratios = torch.from_numpy(np.ascontiguousarray(default_ratios(n_candidates))).to(device)
        self.dsgc_period = max(1, int(dsgc_period))
        self.dsgc_refine = max(0, int(dsgc_refine))
        # log2 of the spacing of the grid's neighbours around a winner: the first refinement spans one grid step each way
        r = default_ratios(n_candidates)
        self.ratio_step = 2.0 * float(np.log2(r[0] / r[1])) if n_candidates > 1 else 1.0
        self.dev_all = torch.zeros(B.MAX_CANDIDATES, dtype=torch.float64, device=device) if self.dsgc_refine else None
        self._j = torch.arange(n_candidates, dtype=torch.float32, device=device) - float(n_candidates // 2)
        self.backward_calls = 0
        self.last_ratios = None
        self.clip = None
        self.deviation = None
        # Stream of seeds of the stochastic rounding (Eq.3): starts at a hash of the layer's name, so that
        # the layers of a model do not share their draws, and advances by one per backward pass.
        self._seed = int(seed) if seed is not None else (zlib.crc32(name.encode()) << 20 if name else 0)
        self._buffers = {}

    def buffers(self, x_shape, dev) -> _LayerBuffers:
        key = (x_shape, str(dev))
        if key not in self._buffers:
            self._buffers[key] = _LayerBuffers(self, x_shape, dev)
        return self._buffers[key]

    def refine_factors(self, width: float) -> torch.Tensor:
        """2^((j - J/2) * width / J), j = 0..J-1, fp32 on the layer's device (factor 1 at j = J/2)."""
        return torch.exp2(self._j * (width / self._j.numel()))

    def next_seed(self) -> int:
        self._seed += 1
        return self._seed

    def forward(self, x):
        keep = torch.is_grad_enabled() and (x.requires_grad or self.weight.requires_grad)
        y = _Int8ConvFn.apply(x, self.weight.view(self.weight_shape), self, keep)
        if self.bias is not None:
            y = y + self.bias.view(1, -1, 1, 1)
        return y

    def dclr_scale(self, alpha: float = 20.0, beta: float = 0.1) -> float:
        """phi(d_c) = max(exp(-alpha d_c), beta) for the last backward pass (reads d_c back)."""
        if self.deviation is None:
            return 1.0
        return B.int8t_dclr_scale(float(self.deviation.item()), alpha, beta)


class Int8Linear(Int8Conv2d):
    """Drop-in for `torch.nn.Linear`: the 8-bit fully connected layer of Sec.3.6 item 1, run as the
    1 x 1 convolution of a 1 x 1 image through the same entry points.  Input (..., in_features)."""

    def __init__(self, in_features, out_features, bias=True, **kw):
        super().__init__(in_features, out_features, 1, bias=bias, **kw)
        self.in_features, self.out_features = in_features, out_features
        self.weight = torch.nn.Parameter(self.weight.data.view(out_features, in_features))    # nn.Linear's shape

    def forward(self, x):
        lead = x.shape[:-1]
        y = super().forward(x.reshape(-1, self.in_features, 1, 1))
        return y.reshape(*lead, self.out_features)


def replace_modules(model: torch.nn.Module, n_candidates: int = 32, dsgc_period: int = 1, skip=(), dsgc_refine: int = 0) -> int:
    """Swaps, in place, every `nn.Conv2d` the library covers (groups 1 or depthwise, dilation 1, zero
    padding) and every `nn.Linear` of `model` for its INT8 counterpart, keeping the parameters (the
    very Parameter objects, so optimizers and state dicts keep working) -- the automatic match and
    replacement of Sec.3.6 item 1.  Modules whose qualified name is in `skip`, and convolutions the
    library does not cover (other group counts, dilation, non-zero padding modes), are left alone.
    Returns the number of modules replaced."""
    count = 0
    for qual, parent in list(model.named_modules()):
        for child_name, m in list(parent.named_children()):
            full = f"{qual}.{child_name}" if qual else child_name
            if full in skip or isinstance(m, Int8Conv2d):
                continue
            new = None
            if isinstance(m, torch.nn.Conv2d):
                ok = (m.dilation == (1, 1) and m.padding_mode == "zeros" and not isinstance(m.padding, str)
                      and (m.groups == 1 or m.groups == m.in_channels == m.out_channels))
                if ok:
                    new = Int8Conv2d(m.in_channels, m.out_channels, m.kernel_size, m.stride, m.padding, m.groups,
                                     bias=False, n_candidates=n_candidates, dsgc_period=dsgc_period, dsgc_refine=dsgc_refine,
                                     device=m.weight.device, name=full)
            elif isinstance(m, torch.nn.Linear):
                new = Int8Linear(m.in_features, m.out_features, bias=False, n_candidates=n_candidates,
                                 dsgc_period=dsgc_period, dsgc_refine=dsgc_refine, device=m.weight.device, name=full)
            if new is None:
                continue
            new.weight = m.weight
            new.bias = m.bias
            new.train(m.training)
            setattr(parent, child_name, new)
            count += 1
    return count


class DclrSGD(torch.optim.SGD):
    """SGD whose learning rate is scaled per INT8 layer by phi(d_c) of that layer's last backward
    pass: Deviation Counteractive LR Scaling, Sec.3.5 Eq.7.  Parameters that belong to no INT8 layer
    (and the fp32 biases) keep the base rate.  `step()` reads all layers' d_c back in ONE copy."""

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

    def deviations(self):
        """d_c of every INT8 layer's last backward pass (0 where none has run), one device-to-host copy."""
        have = [m.deviation for m in self._layers if m.deviation is not None]
        vals = iter(torch.cat(have).cpu().tolist()) if have else iter(())
        return [next(vals) if m.deviation is not None else 0.0 for m in self._layers]

    @torch.no_grad()
    def step(self, closure=None):
        for g, d in zip(self.param_groups, self.deviations()):
            g["lr"] = g["base_lr"] * B.int8t_dclr_scale(d, self.alpha, self.beta)
        for g in self.param_groups[len(self._layers):]:
            g["lr"] = g["base_lr"]
        return super().step(closure)
