"""The autograd plug-in (paper_1912_12607_amd/autograd.py) against the CPU oracle: one forward and
backward pass of Int8Conv2d must give exactly the tensors the oracle's step gives for the same
inputs, seed and candidate ratios; plus a plausibility check against an fp32 convolution and the
Periodic Update bookkeeping."""
import os
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_1912_12607_amd import inputs  # noqa: E402

REL_TOL = 1e-6
DEV_TOL = 1e-9
STO = oracle.ROUND_STOCHASTIC


def _layer(C, K, ks, stride, pad, groups, seed=0, **kw):
    from paper_1912_12607_amd.autograd import Int8Conv2d
    torch.manual_seed(seed)
    return Int8Conv2d(C, K, ks, stride=stride, padding=pad, groups=groups, seed=100, **kw)


@pytest.mark.parametrize("shape", [
    (2, 16, 8, 8, 32, (3, 3), (1, 1), (1, 1), 1),
    (3, 24, 7, 9, 40, (1, 1), (1, 1), (0, 0), 1),
    (2, 12, 9, 9, 12, (3, 3), (1, 1), (1, 1), 12),
    (2, 20, 11, 13, 10, (3, 3), (2, 2), (0, 0), 1),
])
def test_forward_backward_match_oracle(shape):
    N, C, H, W, K, ks, stride, pad, groups = shape
    m = _layer(C, K, ks, stride, pad, groups)
    r = np.random.default_rng(7)
    x = r.standard_normal((N, C, H, W)).astype(np.float32)
    xt = torch.from_numpy(x).cuda().requires_grad_(True)
    y = m(xt)
    dy = (r.standard_t(3, size=tuple(y.shape)) * 1e-3).astype(np.float32)
    y.backward(torch.from_numpy(dy).cuda())
    torch.cuda.synchronize()

    w = m.weight.detach().cpu().numpy()
    od = oracle.make_desc(N, C, H, W, K, ks[0], ks[1], stride, pad, groups)
    xq, sx = oracle.quantize(x)
    wq, sw = oracle.quantize(w)
    seed = 101                                   # the layer's first backward pass draws seed + 1
    o = oracle.dsgc(dy.reshape(-1), inputs.default_ratios(32), mode=STO, seed=seed)
    dyq, sdy = oracle.quantize(dy, c=o["clip"], mode=STO, seed=seed)
    assert m.clip.item() == o["clip"]
    assert abs(m.deviation.item() - o["deviation"]) < DEV_TOL
    assert m.dclr_scale() == oracle.dclr(m.deviation.item())
    for got, want64, s1, s2 in ((y, oracle.conv_fwd(od, xq, wq), sx, sw),
                                (xt.grad, oracle.conv_bwd_data(od, dyq, wq), sdy, sw),
                                (m.weight.grad, oracle.conv_bwd_weight(od, xq, dyq), sx, sdy)):
        want32, ov = oracle.wrap32(want64)
        assert ov == 0
        ref = oracle.dequant(want32, s1, s2)
        g = got.detach().cpu().numpy()
        assert g.shape == ref.shape
        assert np.all(np.abs(g - ref) <= REL_TOL * np.abs(ref))


def test_close_to_fp32_convolution():
    """Plausibility only: the INT8 layer's outputs and gradients point the same way as an fp32
    convolution's (cosine similarity), to within what 8-bit codes allow."""
    m = _layer(32, 48, (3, 3), (1, 1), (1, 1), 1)
    r = np.random.default_rng(3)
    x = torch.from_numpy(r.standard_normal((4, 32, 12, 12)).astype(np.float32)).cuda()
    xa = x.clone().requires_grad_(True)
    xb = x.clone().requires_grad_(True)
    wb = m.weight.detach().clone().requires_grad_(True)
    ya = m(xa)
    yb = torch.nn.functional.conv2d(xb, wb, padding=1)
    dy = torch.from_numpy(r.standard_normal(tuple(ya.shape)).astype(np.float32)).cuda()
    ya.backward(dy)
    yb.backward(dy)
    cos = lambda a, b: float(torch.nn.functional.cosine_similarity(a.detach().flatten(), b.detach().flatten(), dim=0))
    assert cos(ya, yb) > 0.999
    assert cos(xa.grad, xb.grad) > 0.99
    assert cos(m.weight.grad, wb.grad) > 0.99


def test_periodic_update_keeps_clip_between_searches():
    m = _layer(16, 16, (3, 3), (1, 1), (1, 1), 1, dsgc_period=3)
    r = np.random.default_rng(5)
    clips = []
    for it in range(4):
        x = torch.from_numpy(r.standard_normal((2, 16, 8, 8)).astype(np.float32)).cuda().requires_grad_(True)
        y = m(x)
        dy = (r.standard_t(3, size=tuple(y.shape)) * (1e-3 * (it + 1))).astype(np.float32)
        y.backward(torch.from_numpy(dy).cuda())
        clips.append(m.clip.item())
        assert 0.0 <= m.deviation.item() <= 2.0
    assert clips[0] == clips[1] == clips[2]        # searched at pass 0, kept for passes 1 and 2
    assert clips[3] != clips[0]                    # searched again at pass 3 (the gradients have grown)


def test_clip_refinement_descends_and_matches_oracle():
    """dsgc_refine: further sweeps around the winner of the grid (Sec.3.4 learns the clip by descending d_c).  Each
    sweep keeps the previous winner as a candidate, so d_c cannot rise; the last sweep must equal the oracle's search
    over the same candidates, and the candidates must sit inside one grid step around the grid's winner."""
    r = np.random.default_rng(11)
    x = r.standard_normal((2, 16, 10, 10)).astype(np.float32)
    devs = {}
    for refine in (0, 1, 2):
        m = _layer(16, 24, (3, 3), (1, 1), (1, 1), 1, dsgc_refine=refine)
        y = m(torch.from_numpy(x).cuda().requires_grad_(True))
        if refine == 0:
            dy = (r.standard_t(3, size=tuple(y.shape)) * 1e-3).astype(np.float32)
        y.backward(torch.from_numpy(dy).cuda())
        seed = m._seed
        ratios = m.last_ratios.cpu().numpy()
        o = oracle.dsgc(dy, ratios, STO, seed)
        assert m.clip.item() == o["clip"]
        assert abs(m.deviation.item() - o["deviation"]) <= DEV_TOL
        devs[refine] = m.deviation.item()
        if refine == 0:
            grid = o
            assert np.array_equal(ratios, inputs.default_ratios(32))
        else:
            centre = inputs.default_ratios(32)[grid["jstar"]]
            assert ratios.max() <= min(1.0, centre * 2 ** 0.26) and ratios.min() >= centre * 2 ** -0.26
            assert np.all(np.diff(ratios) >= 0)
    assert devs[2] <= devs[1] <= devs[0]
    assert devs[2] < devs[0]                       # a finer grid around the winner does find a better clip here


def test_dclr_sgd_scales_each_layer_by_phi():
    """Eq.7: the update of an INT8 layer's weight is lr * phi(d_c) * gradient with that layer's own d_c;
    other parameters use the plain rate."""
    from paper_1912_12607_amd.autograd import DclrSGD, Int8Conv2d
    torch.manual_seed(1)
    model = torch.nn.Sequential(Int8Conv2d(8, 16, 3, padding=1, seed=5), torch.nn.ReLU(),
                                Int8Conv2d(16, 16, 3, padding=1, groups=16, seed=9),
                                torch.nn.Flatten(), torch.nn.Linear(16 * 6 * 6, 4).cuda())
    opt = DclrSGD(model, lr=0.5)
    x = torch.randn(3, 8, 6, 6, device="cuda")
    loss = model(x).square().sum()
    loss.backward()
    before = [p.detach().clone() for p in model.parameters()]
    grads = [p.grad.detach().clone() for p in model.parameters()]
    opt.step()
    torch.cuda.synchronize()
    layers = [m for m in model.modules() if isinstance(m, Int8Conv2d)]
    phis = [oracle.dclr(m.deviation.item()) for m in layers]
    assert all(0.1 <= p <= 1.0 for p in phis)
    factors = {id(m.weight): p for m, p in zip(layers, phis)}
    for p, b, g in zip(model.parameters(), before, grads):
        lr = 0.5 * factors.get(id(p), 1.0)
        err = (p.detach() - (b - lr * g)).abs().max().item()
        assert err <= 4 * 2.0 ** -24 * (b.abs() + lr * g.abs()).max().item()      # one fp32 rounding each side



def test_int8_linear_matches_oracle_and_bias_stays_fp32():
    """The fully connected counterpart (Sec.3.6 item 1) is the 1x1 convolution of a 1x1 image through the
    same entry points; the bias is added in fp32 to the dequantized result."""
    from paper_1912_12607_amd.autograd import Int8Linear
    torch.manual_seed(2)
    N, Cin, K = 33, 200, 70
    m = Int8Linear(Cin, K, bias=True, seed=100)
    with torch.no_grad():
        m.bias.copy_(torch.randn(K, device="cuda"))
    assert tuple(m.weight.shape) == (K, Cin)
    r = np.random.default_rng(11)
    x = r.standard_normal((N, Cin)).astype(np.float32)
    xt = torch.from_numpy(x).cuda().requires_grad_(True)
    y = m(xt)
    assert tuple(y.shape) == (N, K)
    dy = (r.standard_t(3, size=(N, K)) * 1e-3).astype(np.float32)
    y.backward(torch.from_numpy(dy).cuda())
    torch.cuda.synchronize()
    w = m.weight.detach().cpu().numpy().reshape(K, Cin, 1, 1)
    od = oracle.make_desc(N, Cin, 1, 1, K, 1, 1)
    xq, sx = oracle.quantize(x.reshape(N, Cin, 1, 1))
    wq, sw = oracle.quantize(w)
    o = oracle.dsgc(dy.reshape(-1), inputs.default_ratios(32), mode=STO, seed=101)
    dyq, sdy = oracle.quantize(dy.reshape(N, K, 1, 1), c=o["clip"], mode=STO, seed=101)
    ref_y = oracle.dequant(oracle.wrap32(oracle.conv_fwd(od, xq, wq))[0], sx, sw).reshape(N, K)
    want_y = ref_y + m.bias.detach().cpu().numpy()[None, :]
    assert np.all(np.abs(y.detach().cpu().numpy() - want_y) <= REL_TOL * np.abs(ref_y) + 2.0 ** -23 * np.abs(want_y))
    ref_dx = oracle.dequant(oracle.wrap32(oracle.conv_bwd_data(od, dyq, wq))[0], sdy, sw).reshape(N, Cin)
    ref_dw = oracle.dequant(oracle.wrap32(oracle.conv_bwd_weight(od, xq, dyq))[0], sx, sdy).reshape(K, Cin)
    assert np.all(np.abs(xt.grad.cpu().numpy() - ref_dx) <= REL_TOL * np.abs(ref_dx))
    assert m.weight.grad.shape == (K, Cin)
    assert np.all(np.abs(m.weight.grad.cpu().numpy() - ref_dw) <= REL_TOL * np.abs(ref_dw))
    assert np.allclose(m.bias.grad.cpu().numpy(), dy.sum(0), rtol=1e-5, atol=1e-9)


def test_replace_modules_swaps_conv_and_linear_and_trains_without_new_buffers():
    """The automatic match and replacement (Sec.3.6 item 1): Conv2d (dense and depthwise) and Linear
    become INT8 layers that keep the very Parameter objects; a convolution the library does not cover
    (dilation 2) and a skipped module stay; the replaced model's output and gradients point the same
    way as the fp32 model's; after the first iteration a training loop re-uses every code buffer."""
    from paper_1912_12607_amd.autograd import DclrSGD, Int8Conv2d, Int8Linear, replace_modules
    torch.manual_seed(4)
    nn = torch.nn

    def make():
        return nn.Sequential(nn.Conv2d(3, 16, 3, padding=1, bias=True), nn.ReLU(),
                             nn.Conv2d(16, 16, 3, padding=1, groups=16, bias=False), nn.ReLU(),
                             nn.Conv2d(16, 24, 3, padding=2, dilation=2), nn.ReLU(),
                             nn.Conv2d(24, 32, 1, stride=2), nn.Flatten(),
                             nn.Linear(32 * 5 * 5, 10), nn.ReLU(), nn.Linear(10, 4)).cuda()
    ref = make()
    model = make()
    model.load_state_dict(ref.state_dict())
    params = [id(p) for p in model.parameters()]
    assert replace_modules(model, skip=("10",)) == 4
    assert [type(m).__name__ for m in model] == ["Int8Conv2d", "ReLU", "Int8Conv2d", "ReLU", "Conv2d", "ReLU",
                                                 "Int8Conv2d", "Flatten", "Int8Linear", "ReLU", "Linear"]
    assert [id(p) for p in model.parameters()] == params
    assert set(model.state_dict()) == set(ref.state_dict())
    assert len({m._seed for m in model if isinstance(m, Int8Conv2d)}) == 4       # every layer its own draw stream
    x = torch.randn(6, 3, 10, 10, device="cuda")
    cos = lambda a, b: float(torch.nn.functional.cosine_similarity(a.detach().flatten(), b.detach().flatten(), dim=0))
    ya, yb = model(x), ref(x)
    assert cos(ya, yb) > 0.995
    ya.square().sum().backward()
    yb.square().sum().backward()
    for (n, pa), pb in zip(model.named_parameters(), ref.parameters()):
        assert pa.grad is not None and pa.grad.shape == pb.grad.shape, n
        assert cos(pa.grad, pb.grad) > 0.95, n
    opt = DclrSGD(model, lr=1e-3)
    assert len(opt.deviations()) == 4 and all(0.0 <= d <= 2.0 for d in opt.deviations())
    int8 = [m for m in model if isinstance(m, Int8Conv2d)]
    held = None
    for it in range(4):
        opt.zero_grad()
        model(x).square().sum().backward()
        opt.step()
        bufs = [id(b.ws) for m in int8 for b in m._buffers.values()] + [id(t[0]) for m in int8 for b in m._buffers.values() for t in b.xq_pool]
        assert all(len(m._buffers) == 1 and len(next(iter(m._buffers.values())).xq_pool) == 1 for m in int8)
        if held is not None:
            assert bufs == held                    # same scratch and code buffers as in the previous iteration
        held = bufs
    with torch.no_grad():                          # inference: the activation codes go straight back to the pool
        model(x)
    assert all(len(next(iter(m._buffers.values())).xq_pool) == 1 for m in int8)
