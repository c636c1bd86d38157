"""One conv-layer training step of the INT8 path as a sequence of C-ABI calls.

Pure plumbing: allocates device buffers with torch, uploads the fp32 tensors once, and chains
    quantize_batch(a, W) -> dsgc_clip(g_z) -> quantize(g_z; clip, stochastic, d_c)
    -> conv_fwd -> conv_bwd_data -> conv_bwd_weight
on one stream with no host synchronisation in between (scales, clip and deviation stay in device
memory).  Used by the tests, the smoke check and the benchmark.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from .inputs import Layer


def pad16(v: int) -> int:
    return (v + 15) & ~15


def align256(v: int) -> int:
    return (v + 255) & ~255


def two_stream_default(L: Layer) -> bool:
    """Whether LayerStep.run(overlap=None) uses the second stream in a step that searches the clip: the
    search must be long enough to hide the other chain behind (the hand-over between the streams costs
    about 10 us per step, and the extra calls make a step cost the host about 100 us: over the dense
    layers of ResNet-50, MobileNetV2 and InceptionV3 at batch 32-64 the second stream gains from about
    6 M gradient elements on and loses up to 20 us below 5 M; MobileNetV2's depthwise layers gain from
    7 M elements on: 144 channels at 56 x 56, batch 64, 300 -> 258 us)."""
    return L.N * L.K * L.P * L.Q >= (6 << 20)


_SIDE_STREAMS: dict = {}


def side_stream(device) -> "torch.cuda.Stream":
    """The second stream of the two-stream step, ONE per device for all layers.  The runtime spreads
    streams over a handful of hardware queues (four by default); every further stream shares a queue
    with an earlier one, and a second stream that lands on the main stream's queue runs behind it
    instead of beside it (measured: a fresh stream per layer lost the whole gain on every fourth
    layer).  The first stream created after the main one has a queue of its own."""
    dev = torch.device(device)
    key = dev.index if dev.index is not None else torch.cuda.current_device()
    if key not in _SIDE_STREAMS:
        _SIDE_STREAMS[key] = torch.cuda.Stream(device=dev)
    return _SIDE_STREAMS[key]


class LayerStep:
    def __init__(self, L: Layer, n_cand: int = 32, keep_acc: bool = False, device: str = "cuda:0",
                 requantize_deviation: bool = True, input_grad: bool = True, fused_fwd: bool = False):
        """input_grad=False leaves the backward-data pass out (the first layer of a network: nothing
        consumes the gradient of the images).
        requantize_deviation: also let the quantizer of g_z report Eq.6 for the codes it wrote (into
        dev_final).  The clip search has already returned the same d_c (dev_search), which is what Eq.7
        consumes, so a training step can leave this off."""
        self.L, self.n_cand, self.dev = L, n_cand, torch.device(device)
        # fused_fwd: quantize a inside the forward convolution (int8t_conv_fwd_fused; 1x1 stride-1 layers only)
        self.fused_fwd = bool(fused_fwd)
        if self.fused_fwd:
            assert L.groups == 1 and (L.R, L.S) == (1, 1) and L.stride == (1, 1) and L.pad == (0, 0), "1x1 stride-1 layers"
        self.requantize_deviation = requantize_deviation
        self.input_grad = input_grad
        self.depthwise = L.groups != 1
        self.desc = B.make_desc(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad, L.groups)
        self.act_kind = B.ACT_PLANAR if self.depthwise else B.ACT
        self.wgt_kind = B.WGT_PLANAR if self.depthwise else B.WGT
        d = self.dev
        f32, i8, i32, f64 = torch.float32, torch.int8, torch.int32, torch.float64
        self.x = torch.empty(L.x_shape, dtype=f32, device=d)
        self.w = torch.empty(L.w_shape, dtype=f32, device=d)
        self.dy = torch.empty(L.y_shape, dtype=f32, device=d)
        self.ratios = torch.empty(n_cand, dtype=f32, device=d)
        self.xq = torch.empty(B.int8t_code_bytes(L.x_shape, self.act_kind), dtype=i8, device=d)
        self.wq = torch.empty(B.int8t_code_bytes(L.w_shape, self.wgt_kind), dtype=i8, device=d)
        self.dyq = torch.empty(B.int8t_code_bytes(L.y_shape, self.act_kind), dtype=i8, device=d)
        self.sx = torch.empty(1, dtype=f32, device=d)
        self.sw = torch.empty(1, dtype=f32, device=d)
        self.sdy = torch.empty(1, dtype=f32, device=d)
        self.clip = torch.empty(1, dtype=f32, device=d)
        self.dev_search = torch.empty(1, dtype=f64, device=d)
        self.dev_all = torch.empty(n_cand, dtype=f64, device=d)
        self.dev_final = torch.empty(1, dtype=f64, device=d)
        self.y = torch.empty(L.y_shape, dtype=f32, device=d)
        self.dx = torch.empty(L.x_shape, dtype=f32, device=d)
        self.dw = torch.empty(L.w_shape, dtype=f32, device=d)
        self.y_acc = torch.empty(L.y_shape, dtype=i32, device=d) if keep_acc else None
        self.dx_acc = torch.empty(L.x_shape, dtype=i32, device=d) if keep_acc else None
        self.dw_acc = torch.empty(L.w_shape, dtype=i32, device=d) if keep_acc else None
        n_y = int(np.prod(L.y_shape))
        # one scratch buffer per tensor's chain of calls, so that a caller may put the chains on different streams
        u8 = torch.uint8
        self.ws_x = torch.empty(max(256, B.int8t_quantize_workspace_bytes(L.x_shape, self.act_kind)), dtype=u8, device=d)
        self.ws_w = torch.empty(max(256, B.int8t_quantize_workspace_bytes(L.w_shape, self.wgt_kind)), dtype=u8, device=d)
        self.ws_dy = torch.empty(max(256, B.int8t_quantize_workspace_bytes(L.y_shape, self.act_kind),
                                     B.int8t_workspace_bytes(B.OP_DSGC, None, n_y, n_cand)), dtype=u8, device=d)
        self.ws = torch.empty(max(256, B.int8t_workspace_bytes(B.OP_CONV_BWD_WEIGHT, self.desc)), dtype=u8, device=d)
        # optional scratch of the forward / backward-data passes (split reduction of few-tile layers)
        nf = B.int8t_workspace_bytes(B.OP_CONV_FWD, self.desc)
        nb = B.int8t_workspace_bytes(B.OP_CONV_BWD_DATA, self.desc)
        self.xw_items = [(self.x, L.x_shape, self.act_kind, None, self.xq, self.sx),
                         (self.w, L.w_shape, self.wgt_kind, None, self.wq, self.sw)]
        # (sized for the call that also carries g_z, in the steps that keep the clip value)
        self.ws_xw = torch.empty(B.int8t_quantize_batch_workspace_bytes(
            self.xw_items + [(self.dy, L.y_shape, self.act_kind, self.clip, self.dyq, self.sdy)]), dtype=u8, device=d)
        self._side = None
        self._tuned_overlap = None
        self._tuned_fork = None
        self.ws_fwd = torch.empty(nf, dtype=u8, device=d) if nf else None
        self.ws_bwd_data = torch.empty(nb, dtype=u8, device=d) if nb else None

        self._bind_calls()

    def _bind_calls(self):
        """The calls of run() with their arguments marshalled once (the buffers live as long as the object):
        nine calls with about ten arguments each otherwise cost the host 65 us per step, which is the whole
        step time of a small layer."""
        import ctypes as C
        p, nb, lib, L = B._ptr, B._nbytes, B.lib, self.L
        n_y = self.dy.numel()
        self._items_xw = B._items(self.xw_items)
        self._items_xwg = B._items(self.xw_items + [(self.dy, L.y_shape, self.act_kind, self.clip, self.dyq, self.sdy,
                                                     B.ROUND_STOCHASTIC, 0)])
        self._k_xw = B.bind(lib.int8t_quantize_batch, 2, self._items_xw, p(self.ws_xw), nb(self.ws_xw))
        self._k_xwg = B.bind(lib.int8t_quantize_batch, 3, self._items_xwg, p(self.ws_xw), nb(self.ws_xw))
        self._k_w = B.bind(lib.int8t_quantize, p(self.w), B._dims(L.w_shape), self.wgt_kind, None, B.ROUND_NEAREST_EVEN, 0,
                           p(self.wq), p(self.sw), None, p(self.ws_w), nb(self.ws_w))
        self._k_fwd_fused = B.bind(lib.int8t_conv_fwd_fused, C.byref(self.desc), p(self.x), None, p(self.wq), p(self.sw), p(self.y),
                                   p(self.y_acc), p(self.xq), p(self.sx), p(self.ws_x), nb(self.ws_x))
        self._k_prepare = B.bind(lib.int8t_dsgc_prepare, p(self.dy), n_y, p(self.ws_dy), nb(self.ws_dy))
        self._k_xw_prepare = B.bind(lib.int8t_quantize_batch_prepare, 2, self._items_xw, p(self.ws_xw), nb(self.ws_xw),
                                    p(self.dy), n_y, p(self.ws_dy), nb(self.ws_dy))
        d = C.byref(self.desc)
        self._k_fwd = B.bind(lib.int8t_conv_fwd, d, p(self.xq), p(self.sx), p(self.wq), p(self.sw), p(self.y), p(self.y_acc),
                             p(self.ws_fwd), nb(self.ws_fwd))
        self._k_bwd_data = B.bind(lib.int8t_conv_bwd_data, d, p(self.dyq), p(self.sdy), p(self.wq), p(self.sw), p(self.dx),
                                  p(self.dx_acc), p(self.ws_bwd_data), nb(self.ws_bwd_data))
        self._k_bwd_weight = B.bind(lib.int8t_conv_bwd_weight, d, p(self.xq), p(self.sx), p(self.dyq), p(self.sdy), p(self.dw),
                                    p(self.dw_acc), p(self.ws), nb(self.ws))
        a_search = (p(self.dy), n_y, p(self.ratios), self.n_cand, B.ROUND_STOCHASTIC)
        b_search = (p(self.clip), p(self.dev_search), p(self.dev_all), p(self.ws_dy), nb(self.ws_dy))
        a_qdy = (p(self.dy), B._dims(L.y_shape), self.act_kind, p(self.clip), B.ROUND_STOCHASTIC)
        b_qdy = (p(self.dyq), p(self.sdy), p(self.dev_final if self.requantize_deviation else None), p(self.ws_dy), nb(self.ws_dy))

        def k_search(seed, sp):
            B._check(lib.int8t_dsgc_search(*a_search, seed, *b_search, sp))

        def k_clip(seed, sp):
            B._check(lib.int8t_dsgc_clip(*a_search, seed, *b_search, sp))

        def k_qdy(seed, sp):
            B._check(lib.int8t_quantize(*a_qdy, seed, *b_qdy, sp))

        self._k_search, self._k_clip, self._k_qdy = k_search, k_clip, k_qdy

    def upload(self, x: np.ndarray, w: np.ndarray, dy: np.ndarray, ratios: np.ndarray):
        self.x.copy_(torch.from_numpy(np.ascontiguousarray(x)))
        self.w.copy_(torch.from_numpy(np.ascontiguousarray(w)))
        self.dy.copy_(torch.from_numpy(np.ascontiguousarray(dy)))
        self.ratios.copy_(torch.from_numpy(np.ascontiguousarray(ratios, dtype=np.float32)))

    # -- the individual calls -------------------------------------------------------------------
    def quantize_x(self, stream=None):
        B.int8t_quantize(self.x, self.L.x_shape, self.act_kind, None, B.ROUND_NEAREST_EVEN, 0,
                         self.xq, self.sx, None, self.ws_x, stream)

    def quantize_w(self, stream=None):
        B.int8t_quantize(self.w, self.L.w_shape, self.wgt_kind, None, B.ROUND_NEAREST_EVEN, 0,
                         self.wq, self.sw, None, self.ws_w, stream)

    def quantize_xw(self, stream=None):
        """a and W in one batched call: same codes and scales as quantize_x() + quantize_w()."""
        B.int8t_quantize_batch(self.xw_items, self.ws_xw, stream)

    def dsgc(self, seed: int, stream=None):
        B.int8t_dsgc_clip(self.dy, self.dy.numel(), self.ratios, self.n_cand, B.ROUND_STOCHASTIC, seed,
                          self.clip, self.dev_search, self.dev_all, self.ws_dy, stream)

    def quantize_dy(self, seed: int, stream=None):
        B.int8t_quantize(self.dy, self.L.y_shape, self.act_kind, self.clip, B.ROUND_STOCHASTIC, seed,
                         self.dyq, self.sdy, self.dev_final if self.requantize_deviation else None, self.ws_dy, stream)

    def fwd(self, stream=None):
        B.int8t_conv_fwd(self.desc, self.xq, self.sx, self.wq, self.sw, self.y, self.y_acc, self.ws_fwd, stream)

    def bwd_data(self, stream=None):
        if not self.input_grad:
            return
        B.int8t_conv_bwd_data(self.desc, self.dyq, self.sdy, self.wq, self.sw, self.dx, self.dx_acc,
                              self.ws_bwd_data, stream)

    def bwd_weight(self, stream=None):
        B.int8t_conv_bwd_weight(self.desc, self.xq, self.sx, self.dyq, self.sdy, self.dw, self.dw_acc,
                                self.ws, stream)

    def run(self, seed: int = 0, stream=None, search: bool = True, overlap: bool | int | None = False):
        """The whole hot path once.  search=False keeps the clip value of the last search (the
        paper's Periodic Update, Sec.3.4 / Table 2: the clip is refreshed every P iterations only);
        the caller decides the period.

        overlap chooses the schedule of the same calls on the caller's stream and a second one (both
        of the default priority; outputs are complete once the caller's stream is):
          False / 0  everything on one stream;
          True / 1   the quantization of a and W and the forward convolution on the second stream
                     beside the clip search: the two chains are independent until the backward
                     convolutions, the search is bound by the vector ALUs and the other kernels by HBM;
          2          one stream up to the codes, then backward-weight on the second stream beside the
                     forward and backward-data convolutions: the three passes depend only on the codes,
                     and on layers whose tiles do not fill the chip they run beside each other;
          3          both: backward-weight follows the forward pass on the second stream, and backward-data
                     starts as soon as the codes of W are there, beside the forward pass if that is still running;
          4          as 1, but the backward passes wait for the codes of a and W only, not for the forward pass
                     behind them (with 1 each convolution has the chip to itself).
        A step that keeps the clip has no search to hide anything behind: any non-zero value means 2.
        overlap=None follows tune() if it has run, else two_stream_default() in steps that search
        and one stream in steps that do not."""
        if overlap is None:
            if search:
                overlap = self._tuned_overlap if self._tuned_overlap is not None else two_stream_default(self.L)
            else:
                overlap = self._tuned_fork or 0
        mode = int(overlap)
        batched = not search and not self.requantize_deviation and not self.fused_fwd
        if mode and batched:
            mode = 2
        if not mode:
            sp = B.stream_pointer(stream)
            if batched:
                # the clip value is known: a, W and g_z in one batched call (one launch fewer)
                self._items_xwg[2].seed = seed
                self._k_xwg(sp)
            elif self.fused_fwd:
                self._k_w(sp)
                if search:
                    self._k_clip(seed, sp)
                self._k_qdy(seed, sp)
            elif search:
                # max|.| of a, W and g_z (with the sums the search needs) in one launch, then the sweep
                self._k_xw_prepare(sp)
                self._k_search(seed, sp)
                self._k_qdy(seed, sp)
            else:
                self._k_xw(sp)
                self._k_qdy(seed, sp)
            if self.fused_fwd:
                self._k_fwd_fused(sp)
            else:
                self._k_fwd(sp)
            if self.input_grad:
                self._k_bwd_data(sp)
            self._k_bwd_weight(sp)
            return
        main = stream if stream is not None else torch.cuda.current_stream()
        if self._side is None:
            self._side = side_stream(self.dev)
            self._ev_main, self._ev_main2, self._ev_side, self._ev_side2 = (torch.cuda.Event() for _ in range(4))
        side = self._side
        mp, sp = B.stream_pointer(main), B.stream_pointer(side)
        if mode == 2:
            if batched:
                self._items_xwg[2].seed = seed
                self._k_xwg(mp)
            else:
                if search and not self.fused_fwd:
                    self._k_xw_prepare(mp)
                    self._k_search(seed, mp)
                else:
                    (self._k_w if self.fused_fwd else self._k_xw)(mp)
                    if search:
                        self._k_clip(seed, mp)
                self._k_qdy(seed, mp)
                if self.fused_fwd:
                    self._k_fwd_fused(mp)       # writes the codes of a, which backward-weight reads
            self._ev_main.record(main)
            side.wait_event(self._ev_main)
            self._k_bwd_weight(sp)
            self._ev_side.record(side)
            if not self.fused_fwd:
                self._k_fwd(mp)
            if self.input_grad:
                self._k_bwd_data(mp)
            main.wait_event(self._ev_side)
            return
        # main stream: clip search, quantize g_z, then backward-data (and backward-weight, unless it is forked).
        # side stream: quantize a and W, forward convolution (needs nothing from the gradient chain).
        # It starts behind whatever is queued on the main stream up to the search's first pass (the
        # previous step's backward passes still read the codes that are about to be overwritten, and
        # that pass is bound by HBM like the side stream's kernels: beside each other they would only
        # slow each other down), i.e. together with the sweep.
        if search:
            self._k_prepare(mp)
        self._ev_main.record(main)
        side.wait_event(self._ev_main)
        early = mode >= 3 and not self.fused_fwd
        if self.fused_fwd:
            self._k_w(sp)
            self._k_fwd_fused(sp)               # writes the codes of a
            self._ev_side.record(side)
        else:
            self._k_xw(sp)
            if early:
                self._ev_side.record(side)      # the codes of a and W are there
            self._k_fwd(sp)
            if not early:
                self._ev_side.record(side)
        if search:
            self._k_search(seed, mp)
        self._k_qdy(seed, mp)
        if mode == 3:
            # backward-weight follows the forward pass on the side stream once g_z has its codes
            self._ev_main2.record(main)
            side.wait_event(self._ev_main2)
            self._k_bwd_weight(sp)
        if early or mode == 3:
            self._ev_side2.record(side)
        main.wait_event(self._ev_side)
        if self.input_grad:
            self._k_bwd_data(mp)
        if mode != 3:
            self._k_bwd_weight(mp)
        if early or mode == 3:
            main.wait_event(self._ev_side2)

    def tune(self, steps: int = 40) -> int:
        """Choose the schedule (run()'s overlap values) by timing them on this layer's own buffers (the
        per-layer choice "before training" of the paper's Suppl. "INT8 Convolution", here between schedules of
        the same kernels): once for steps that search the clip and once for steps that keep it.
        run(overlap=None) then follows the measurement.  Returns the choice for searching steps.  The buffers
        must hold data (upload() first; the steps that keep the clip quantize with whatever the clip buffer
        holds, so a searching step should have run); their contents are what a step leaves."""
        import time

        def timed(search, overlap):
            for k in range(steps):
                self.run(seed=k, search=search, overlap=overlap)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for k in range(steps):
                self.run(seed=k, search=search, overlap=overlap)
            torch.cuda.synchronize()
            return time.perf_counter() - t0

        self._tuned_fork = min((0, 2), key=lambda m: timed(False, m))
        self._tuned_overlap = min((0, 1, 2, 3, 4), key=lambda m: timed(True, m))
        return self._tuned_overlap

    def refresh_scratch(self):
        """Re-size the backward-weight scratch after a kernel selection made elsewhere for this shape (the
        selection is per shape and process-wide; the scratch of that pass depends on it)."""
        need = B.int8t_workspace_bytes(B.OP_CONV_BWD_WEIGHT, self.desc)
        if need > self.ws.numel():
            self.ws = torch.empty(need, dtype=torch.uint8, device=self.dev)
            self._bind_calls()

    def tune_kernels(self, reps: int = 30, verbose: bool = False) -> dict:
        """The per-layer choice of the convolution kernels "before training" (Suppl. "INT8 Convolution",
        last paragraph): for each of the three passes, times every kernel variant the library admits for
        this layer on the layer's own buffers and selects the fastest (int8t_conv_select_variant; the
        library keeps the choice per (pass, shape), so every layer of that shape in the process uses it).
        All variants write identical results.  The code buffers must hold codes (run() once before).
        Returns {pass: (chosen variant name, {variant name: microseconds})}."""
        import time
        if self.depthwise:
            return {}
        out = {}
        for name, op, call in (("fwd", B.OP_CONV_FWD, "_k_fwd"), ("bwd_data", B.OP_CONV_BWD_DATA, "_k_bwd_data"),
                               ("bwd_weight", B.OP_CONV_BWD_WEIGHT, "_k_bwd_weight")):
            if name == "bwd_data" and not self.input_grad:
                continue
            times = {}
            sp = B.stream_pointer(None)
            for v in range(len(B.VARIANT_NAMES)):
                if not B.int8t_conv_variant_ok(op, self.desc, v):
                    continue
                B.int8t_conv_select_variant(op, self.desc, v)
                if op == B.OP_CONV_BWD_WEIGHT:
                    need = B.int8t_workspace_bytes(op, self.desc)      # depends on the variant's split count
                    if need > self.ws.numel():
                        self.ws = torch.empty(need, dtype=torch.uint8, device=self.dev)
                        self._bind_calls()
                fn = getattr(self, call)
                for _ in range(5):
                    fn(sp)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(reps):
                    fn(sp)
                torch.cuda.synchronize()
                times[v] = (time.perf_counter() - t0) / reps * 1e6
            # the library's own choice stays unless another variant is at least 2 % faster (timing noise)
            best = min(times, key=times.get)
            if times[best] > 0.98 * times[B.VARIANT_AUTO]:
                best = B.VARIANT_AUTO
            B.int8t_conv_select_variant(op, self.desc, best)
            if op == B.OP_CONV_BWD_WEIGHT:
                need = B.int8t_workspace_bytes(op, self.desc)
                if need > self.ws.numel():
                    self.ws = torch.empty(need, dtype=torch.uint8, device=self.dev)
                    self._bind_calls()
            out[name] = (B.VARIANT_NAMES[best], {B.VARIANT_NAMES[v]: round(t, 2) for v, t in times.items()})
            if verbose:
                print(self.L.name, name, out[name], flush=True)
        return out

    # -- host copies of the code tensors in logical order (the library's own unpacking aid) ----------
    def codes_x(self) -> np.ndarray:
        return unpack_act(self.xq.cpu().numpy(), self.L.x_shape, self.depthwise)

    def codes_dy(self) -> np.ndarray:
        return unpack_act(self.dyq.cpu().numpy(), self.L.y_shape, self.depthwise)

    def codes_w(self):
        return unpack_wgt(self.wq.cpu().numpy(), self.L.w_shape, self.depthwise)


def unpack_act(q: np.ndarray, shape, planar: bool) -> np.ndarray:
    """Library layout -> logical N,C,H,W codes (int8t_unpack_codes).  Checks that channel padding is zero."""
    out, bad = B.int8t_unpack_codes(q, shape, B.ACT_PLANAR if planar else B.ACT)
    assert bad == 0, "channel padding of the code tensor must be zero"
    return out


def unpack_wgt(q: np.ndarray, shape, planar: bool):
    """Library layout -> (logical K,Cg,R,S codes, same from the backward-data copy or None)."""
    if planar:
        return B.int8t_unpack_codes(q, shape, B.WGT_PLANAR)[0], None
    a, bad_a = B.int8t_unpack_codes(q, shape, B.WGT, 0)
    b, bad_b = B.int8t_unpack_codes(q, shape, B.WGT, 1)
    assert bad_a == 0 and bad_b == 0, "padding of the weight codes must be zero"
    return a, b
