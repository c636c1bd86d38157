"""GPU parity: every C-ABI call against the CPU oracle, element by element, on seeded inputs.

Bars: int8 codes and int32 accumulators bit-exact; dequantized fp32 outputs within 1e-6 relative
(three fp32 roundings on the GPU -- int32->fp32, s_a*s_b, the product -- against one rounding of
the exact double product in the oracle: <= 3 * 2^-24 = 1.8e-7); direction deviations within 1e-9
absolute (both sides sum in fp64, only the order differs: error <= n * 2^-53 relative to sums
whose ratio is <= 1).
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import oracle  # noqa: E402
from paper_1912_12607_amd import binding as B  # noqa: E402
from paper_1912_12607_amd import inputs  # noqa: E402
from paper_1912_12607_amd.step import LayerStep, align256, pad16, unpack_act, unpack_wgt  # noqa: E402

DEV = torch.device("cuda:0")
RTN, STO = B.ROUND_NEAREST_EVEN, B.ROUND_STOCHASTIC
DEV_TOL = 1e-9
REL_TOL = 1e-6


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def pack_act(q):
    N, C, H, W = q.shape
    out = np.zeros((N, H, W, pad16(C)), np.int8)
    out[..., :C] = q.transpose(0, 2, 3, 1)
    return out.reshape(-1)


def pack_wgt(w):
    K, Cg, R, S = w.shape
    Cp, Kp = pad16(Cg), pad16(K)
    n1 = K * R * S * Cp
    buf = np.zeros(align256(n1) + Cg * R * S * Kp, np.int8)
    a = np.zeros((K, R, S, Cp), np.int8)
    a[..., :Cg] = w.transpose(0, 2, 3, 1)
    b = np.zeros((Cg, R, S, Kp), np.int8)
    b[..., :K] = w.transpose(1, 2, 3, 0)
    buf[:n1] = a.reshape(-1)
    buf[align256(n1):] = b.reshape(-1)
    return buf


def gpu_quantize(x, kind, clip=None, mode=RTN, seed=0, want_dev=False):
    x = np.ascontiguousarray(x, np.float32)
    dims = x.shape
    xd = dev(x)
    q = torch.full((B.int8t_code_bytes(dims, kind),), 77, dtype=torch.int8, device=DEV)
    s = torch.zeros(1, dtype=torch.float32, device=DEV)
    d = torch.zeros(1, dtype=torch.float64, device=DEV) if want_dev else None
    ws = torch.empty(max(B.int8t_quantize_workspace_bytes(dims, kind), 256), dtype=torch.uint8, device=DEV)
    cd = dev(np.array([clip], np.float32)) if clip is not None else None
    B.int8t_quantize(xd, dims, kind, cd, mode, seed, q, s, d, ws)
    torch.cuda.synchronize()
    return q.cpu().numpy(), np.float32(s.item()), (d.item() if want_dev else None)


ACT_SHAPES = [(2, 16, 16, 16), (1, 3, 5, 7), (3, 24, 14, 14), (2, 70, 17, 17), (1, 144, 9, 3),
              (2, 64, 8, 8), (1, 1, 1, 1), (5, 130, 1, 66),
              (33, 208, 1, 1), (7, 200, 1, 1)]      # 1 x 1 images: without / with channel padding


@pytest.mark.parametrize("shape", ACT_SHAPES)
@pytest.mark.parametrize("mode", [RTN, STO])
def test_quantize_act_bit_exact(shape, mode):
    r = np.random.RandomState(hash(shape) % 1000)
    x = r.standard_normal(shape).astype(np.float32) * 3
    for clip in (None, 2.5):
        q, s, d = gpu_quantize(x, B.ACT, clip, mode, seed=11, want_dev=True)
        qo, so = oracle.quantize(x, c=clip, mode=mode, seed=11)
        assert s == so
        assert np.array_equal(unpack_act(q, shape, False), qo)
        assert abs(d - oracle.deviation(x, qo, so)) < DEV_TOL


def test_quantize_act_ties_and_representable():
    k = np.arange(-127, 128, dtype=np.int32)
    x = np.zeros((1, 5, 17, 15), np.float32)
    x.reshape(-1)[:255] = k * 0.5
    x.reshape(-1)[300:308] = [0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, 62.5]
    q, s, _ = gpu_quantize(x, B.ACT, clip=127.0)
    qo, so = oracle.quantize(x, c=127.0)
    assert np.array_equal(unpack_act(q, x.shape, False), qo) and s == so == 1.0


@pytest.mark.parametrize("shape", [(32, 16, 3, 3), (5, 3, 1, 7), (24, 144, 1, 1), (70, 33, 3, 3)])
@pytest.mark.parametrize("mode", [RTN, STO])
def test_quantize_wgt_both_copies(shape, mode):
    w = (np.random.RandomState(3).standard_normal(shape) * 0.1).astype(np.float32)
    q, s, d = gpu_quantize(w, B.WGT, None, mode, seed=5, want_dev=True)
    qo, so = oracle.quantize(w, mode=mode, seed=5)
    a, b = unpack_wgt(q, shape, False)
    assert s == so and np.array_equal(a, qo) and np.array_equal(b, qo)
    assert abs(d - oracle.deviation(w, qo, so)) < DEV_TOL


@pytest.mark.parametrize("shape", [(2, 4, 5, 5), (1, 3, 7, 9), (3, 144, 14, 14), (1, 1, 1, 3)])
@pytest.mark.parametrize("mode", [RTN, STO])
def test_quantize_planar(shape, mode):
    x = np.random.RandomState(4).standard_normal(shape).astype(np.float32)
    for kind in (B.ACT_PLANAR, B.WGT_PLANAR):
        q, s, d = gpu_quantize(x, kind, None, mode, seed=2 ** 40 + 9, want_dev=True)
        qo, so = oracle.quantize(x, mode=mode, seed=2 ** 40 + 9)
        assert s == so and np.array_equal(q.reshape(shape), qo)
        assert abs(d - oracle.deviation(x, qo, so)) < DEV_TOL


def test_quantize_random_shapes():
    """Seeded random tensors in every layout (narrow and wide channel counts, 1 x 1 images, filters of 1 to
    49 taps with ragged filter / channel counts), both rounding modes, with and without a clip value:
    codes, scale and deviation against the oracle."""
    r = np.random.RandomState(5)
    for it in range(90):
        kind = [B.ACT, B.WGT, B.ACT_PLANAR][it % 3]
        if kind == B.WGT:
            R, S = int(r.choice([1, 1, 2, 3, 7])), int(r.choice([1, 1, 3, 5, 7]))
            shape = (int(r.choice([1, 5, 16, 17, 70, 130])), int(r.choice([1, 3, 16, 33, 64, 100, 200])), R, S)
        else:
            H, W = (1, 1) if r.rand() < 0.25 else (int(r.randint(1, 20)), int(r.randint(1, 20)))
            shape = (int(r.randint(1, 6)), int(r.choice([1, 3, 16, 17, 48, 64, 130, 208])), H, W)
        mode = STO if r.rand() < 0.5 else RTN
        clip = None if r.rand() < 0.5 else float(r.uniform(0.5, 3.0))
        seed = int(r.randint(0, 2 ** 31))
        x = (r.standard_normal(shape) * 2).astype(np.float32)
        q, s, d = gpu_quantize(x, kind, clip, mode, seed=seed, want_dev=True)
        qo, so = oracle.quantize(x, c=clip, mode=mode, seed=seed)
        assert s == so, (shape, kind, mode, clip)
        if kind == B.ACT:
            got = unpack_act(q, shape, False)
        elif kind == B.WGT:
            got, got2 = unpack_wgt(q, shape, False)
            assert np.array_equal(got2, qo), (shape, kind, mode, clip)
        else:
            got = q.reshape(shape)
        assert np.array_equal(got, qo), (shape, kind, mode, clip)
        assert abs(d - oracle.deviation(x, qo, so)) < DEV_TOL, (shape, kind, mode, clip)


def test_quantize_zero_tensor_and_nan():
    z = np.zeros((2, 5, 4, 4), np.float32)
    for mode in (RTN, STO):
        q, s, d = gpu_quantize(z, B.ACT, None, mode, seed=1, want_dev=True)
        assert not q.any() and s == 0.0 and d == 0.0
    x = np.random.RandomState(1).standard_normal((1, 16, 4, 4)).astype(np.float32)
    x[0, 3, 2, 1] = np.nan
    q, s, _ = gpu_quantize(x, B.ACT)
    qo, so = oracle.quantize(x)
    assert s == so and np.array_equal(unpack_act(q, x.shape, False), qo) and qo[0, 3, 2, 1] == 0


def gpu_dsgc(g, ratios, mode, seed):
    g = np.ascontiguousarray(g, np.float32).reshape(-1)
    J = len(ratios)
    clip = torch.zeros(1, dtype=torch.float32, device=DEV)
    d = torch.zeros(1, dtype=torch.float64, device=DEV)
    da = torch.zeros(J, dtype=torch.float64, device=DEV)
    ws = torch.empty(B.int8t_workspace_bytes(B.OP_DSGC, None, g.size, J), dtype=torch.uint8, device=DEV)
    B.int8t_dsgc_clip(dev(g), g.size, dev(np.asarray(ratios, np.float32)), J, mode, seed, clip, d, da, ws)
    torch.cuda.synchronize()
    return np.float32(clip.item()), d.item(), da.cpu().numpy()


def check_dsgc(g, ratios, mode, seed):
    clip, d, da = gpu_dsgc(g, ratios, mode, seed)
    o = oracle.dsgc(np.asarray(g, np.float32).reshape(-1), ratios, mode=mode, seed=seed)
    assert np.all(np.abs(da - o["dev"]) < DEV_TOL)
    # several candidates may tie within rounding of the fp64 sums: accept the GPU's winner iff the
    # oracle's deviation at it is within tolerance of the oracle's minimum, and the clip is that candidate's
    j = int(np.argmin(np.abs(o["clips"] - clip)))
    assert clip == o["clips"][j]
    assert o["dev"][j] - o["deviation"] <= 2 * DEV_TOL
    assert abs(d - o["dev"][j]) < DEV_TOL
    return o, j


@pytest.mark.parametrize("n", [1, 3, 1000, 16384, 100003])
@pytest.mark.parametrize("mode", [RTN, STO])
def test_dsgc_small(n, mode):
    r = np.random.RandomState(n % 97)
    g = (r.standard_t(3, size=n) * 1e-3).astype(np.float32)
    if n > 100:
        g[r.choice(n, max(1, n // 10000), replace=False)] *= 100
    check_dsgc(g, inputs.default_ratios(32), mode, seed=n)


def test_dsgc_random_cases():
    """Seeded random lengths (incl. n mod 4 != 0 and lengths around the block / wave sizes), value
    distributions, candidate sets (random, unsorted ratios) and seeds."""
    r = np.random.RandomState(17)
    sizes = [2, 5, 63, 64, 65, 255, 257, 1023, 4097, 65537, 262145] + [int(v) for v in r.randint(6, 300000, size=9)]
    for n in sizes:
        kind = r.randint(3)
        if kind == 0:
            g = (r.standard_t(2, size=n) * 10.0 ** r.uniform(-6, 1)).astype(np.float32)
        elif kind == 1:
            g = r.standard_normal(n).astype(np.float32)
        else:
            g = (r.uniform(-1, 1, size=n) * (r.rand(n) < 0.05)).astype(np.float32)       # mostly zeros
            g[r.randint(n)] = 0.75
        J = int(r.choice([1, 2, 5, 32, 40]))
        ratios = r.uniform(0.01, 1.0, size=J).astype(np.float32)
        mode = STO if r.rand() < 0.6 else RTN
        check_dsgc(g, ratios, mode, seed=int(r.randint(0, 2 ** 31)))


def test_dsgc_candidate_counts_and_degenerate():
    r = np.random.RandomState(5)
    g = (r.standard_t(3, size=50000) * 1e-3).astype(np.float32)
    for J in (1, 7, 33, 64):
        ratios = np.exp2(-np.arange(J) / 8.0).astype(np.float32)
        check_dsgc(g, ratios, STO, seed=3)
    clip, d, da = gpu_dsgc(np.zeros(1000, np.float32), [1.0, 0.5], STO, 1)
    assert clip == 0.0 and d == 0.0 and not da.any()
    # representable inputs, ratio 1: zero deviation
    k = r.randint(-127, 128, size=4096)
    k[0] = 127
    g = (k * 2.0 ** -12).astype(np.float32)
    clip, d, da = gpu_dsgc(g, [1.0, 0.5], STO, 9)
    assert clip == np.float32(127 * 2.0 ** -12) and abs(d) < 1e-15


def test_quantize_batch_prepare_equals_the_two_calls():
    """The batched quantize call that also runs the first phase of a clip search, followed by the sweep, writes
    what int8t_quantize_batch and int8t_dsgc_clip write: codes, scales, clip value and every deviation."""
    r = np.random.RandomState(12)
    x = r.standard_normal((3, 20, 9, 9)).astype(np.float32)
    w = (r.standard_normal((24, 20, 3, 3)) * 0.1).astype(np.float32)
    for n in (5, 4099, 300000):
        g = (r.standard_t(3, n) * 1e-3).astype(np.float32)
        gd, ratios = dev(g), dev(inputs.default_ratios(32))
        outs = []
        for merged in (False, True):
            items = []
            for t, kind in ((x, B.ACT), (w, B.WGT)):
                items.append((dev(t), t.shape, kind, None, torch.full((B.int8t_code_bytes(t.shape, kind),), 77, dtype=torch.int8, device=DEV),
                              torch.zeros(1, dtype=torch.float32, device=DEV), RTN, 0))
            ws = torch.empty(B.int8t_quantize_batch_workspace_bytes(items), dtype=torch.uint8, device=DEV)
            dws = torch.full((B.int8t_workspace_bytes(B.OP_DSGC, None, n, 32),), 0x5A, dtype=torch.uint8, device=DEV)
            clip = torch.zeros(1, dtype=torch.float32, device=DEV)
            d = torch.zeros(1, dtype=torch.float64, device=DEV)
            da = torch.zeros(32, dtype=torch.float64, device=DEV)
            if merged:
                B.int8t_quantize_batch_prepare(items, ws, gd, n, dws)
                B.int8t_dsgc_search(gd, n, ratios, 32, STO, 9, clip, d, da, dws)
            else:
                B.int8t_quantize_batch(items, ws)
                B.int8t_dsgc_clip(gd, n, ratios, 32, STO, 9, clip, d, da, dws)
            torch.cuda.synchronize()
            outs.append([items[0][4], items[0][5], items[1][4], items[1][5], clip, d, da])
        for a, b in zip(*outs):
            assert torch.equal(a, b)
        want = oracle.dsgc(g, inputs.default_ratios(32), mode=STO, seed=9)
        assert np.float32(outs[1][4].item()) == want["clip"] and abs(outs[1][5].item() - want["deviation"]) < DEV_TOL


def test_quantize_batch_equals_single_calls_and_oracle():
    """One batched call = the per-tensor calls, bit for bit (codes, scales), for every layout, with and
    without a supplied clip value."""
    r = np.random.RandomState(11)
    specs = [((3, 20, 6, 6), B.ACT, None),            # H*W a multiple of 4
             ((2, 7, 5, 3), B.ACT, None),             # H*W = 15: one pixel per lane
             ((40, 24, 3, 3), B.WGT, None),
             ((2, 9, 7, 7), B.ACT_PLANAR, 0.75),
             ((130, 70, 1, 1), B.WGT, 1.5),
             # stochastic items (Eq.3): every layout, with and without a clip value
             ((2, 24, 6, 6), B.ACT, 1.25, 99), ((3, 3, 5, 7), B.ACT, None, 7), ((2, 5, 4, 4), B.ACT_PLANAR, None, 5)]
    assert len(specs) == B.MAX_BATCH
    items, singles, host = [], [], []
    for shape, kind, clip, *sd in specs:
        mode, seed = (STO, sd[0]) if sd else (RTN, 0)
        x = (r.standard_normal(shape) * (1.0 + len(host))).astype(np.float32)
        xd = dev(x)
        cd = None if clip is None else dev(np.array([clip], np.float32))
        nq = B.int8t_code_bytes(shape, kind)
        qa, qb = (torch.full((nq,), 77, dtype=torch.int8, device=DEV) for _ in range(2))
        sa, sb = (torch.full((1,), -1.0, dtype=torch.float32, device=DEV) for _ in range(2))
        items.append((xd, shape, kind, cd, qa, sa, mode, seed))
        singles.append((xd, shape, kind, cd, qb, sb, mode, seed))
        host.append((x, clip, mode, seed))
    ws = torch.empty(B.int8t_quantize_batch_workspace_bytes(items), dtype=torch.uint8, device=DEV)
    B.int8t_quantize_batch(items, ws)
    for xd, shape, kind, cd, qb, sb, mode, seed in singles:
        w1 = torch.empty(max(256, B.int8t_quantize_workspace_bytes(shape, kind)), dtype=torch.uint8, device=DEV)
        B.int8t_quantize(xd, shape, kind, cd, mode, seed, qb, sb, None, w1)
    torch.cuda.synchronize()
    for (xd, shape, kind, cd, qa, sa, _, _), (_, _, _, _, qb, sb, _, _), (x, clip, mode, seed) in zip(items, singles, host):
        assert torch.equal(qa, qb) and torch.equal(sa, sb), (shape, kind)
        want_q, want_s = oracle.quantize(x, c=clip, mode=mode, seed=seed)
        assert sa.item() == want_s
        if kind == B.ACT:
            assert np.array_equal(unpack_act(qa.cpu().numpy(), shape, False), want_q)
        elif kind == B.WGT:
            got, got2 = unpack_wgt(qa.cpu().numpy(), shape, False)
            assert np.array_equal(got, want_q) and np.array_equal(got2, want_q)
        else:
            assert np.array_equal(qa.cpu().numpy().reshape(shape), want_q)


# (N, C, H, W, K, R, S, stride, pad, groups)
CONV_SHAPES = [
    (2, 16, 16, 16, 32, 3, 3, (1, 1), (1, 1), 1),
    (1, 3, 5, 5, 4, 3, 3, (1, 1), (1, 1), 1),
    (2, 24, 9, 9, 144, 1, 1, (1, 1), (0, 0), 1),
    (2, 144, 7, 7, 24, 1, 1, (1, 1), (0, 0), 1),
    (1, 20, 11, 13, 70, 3, 3, (2, 2), (0, 0), 1),
    (2, 33, 8, 9, 17, 3, 3, (2, 1), (1, 0), 1),
    (1, 48, 9, 17, 40, 1, 7, (1, 1), (0, 3), 1),
    (1, 48, 17, 9, 40, 7, 1, (1, 1), (3, 0), 1),
    (3, 64, 14, 14, 130, 3, 3, (1, 1), (1, 1), 1),
    (2, 130, 6, 6, 200, 3, 3, (1, 1), (1, 1), 1),
    (1, 8, 12, 12, 8, 5, 5, (3, 2), (2, 2), 1),
    (2, 12, 9, 9, 12, 3, 3, (1, 1), (1, 1), 12),      # depthwise
    (1, 5, 11, 8, 5, 3, 3, (2, 2), (1, 1), 5),        # depthwise stride 2
    (2, 7, 6, 9, 7, 5, 3, (1, 2), (2, 0), 7),         # depthwise odd filter
    (2, 20, 14, 18, 20, 3, 3, (2, 2), (1, 1), 20),    # depthwise stride 2, larger planes
    (1, 6, 13, 10, 6, 5, 5, (3, 3), (2, 2), 6),       # depthwise stride 3 under a 5 x 5 filter
    (1, 3, 9, 9, 3, 2, 2, (3, 2), (0, 1), 3),         # depthwise, stride above the filter height
    (2, 9, 16, 24, 9, 3, 3, (2, 2), (1, 1), 9),       # depthwise stride 2: row length a multiple of 4 (16-byte stores)
    (1, 4, 15, 13, 4, 5, 5, (2, 2), (2, 2), 4),       # 5 x 5 at stride 2, odd sizes
    (1, 4, 12, 12, 4, 5, 5, (2, 2), (1, 2), 4),       # odd and even padding
    (2, 3, 10, 9, 3, 3, 3, (2, 2), (0, 0), 3),        # no padding
    (1, 2, 9, 12, 2, 4, 6, (2, 2), (1, 2), 2),        # even filter at stride 2 (forward fast path, generic backward)
    (33, 200, 1, 1, 70, 1, 1, (1, 1), (0, 0), 1),     # fully connected layer: 1x1 filter on a 1x1 image
    (2, 6, 8, 12, 6, 3, 5, (1, 1), (1, 2), 6),         # depthwise stride 1, 5-wide filter, row length a multiple of 4
    (1, 4, 10, 11, 4, 3, 3, (1, 1), (0, 0), 4),        # depthwise stride 1, no padding
    (3, 5, 16, 16, 5, 3, 3, (1, 1), (1, 1), 5),        # depthwise, plane size a multiple of 16
    # small depthwise planes: a block takes several consecutive planes (whole and partial groups, aligned and not)
    (3, 20, 7, 7, 20, 3, 3, (1, 1), (1, 1), 20),
    (2, 10, 14, 14, 10, 3, 3, (1, 1), (1, 1), 10),
    (2, 10, 14, 14, 10, 3, 3, (2, 2), (1, 1), 10),
    (2, 9, 7, 7, 9, 5, 5, (1, 1), (2, 2), 9),
    (1, 7, 28, 28, 7, 3, 3, (1, 1), (1, 1), 7),
    # ... backward-weight with several channels per block and several images per pass
    (3, 32, 7, 7, 32, 3, 3, (1, 1), (1, 1), 32),
    (2, 12, 14, 14, 12, 3, 3, (1, 1), (1, 1), 12),
    (2, 16, 7, 7, 16, 5, 5, (1, 1), (2, 2), 16),
    (2, 8, 12, 10, 8, 3, 3, (1, 1), (0, 1), 8),        # gradient plane smaller than the input plane
    (64, 384, 14, 14, 384, 3, 3, (1, 1), (1, 1), 384), # a share of more images than one pass stages
    # small filter banks with an even number of channel granules (weights held in registers)
    (2, 64, 7, 20, 64, 3, 3, (1, 1), (1, 1), 1),
    (3, 32, 9, 13, 40, 3, 3, (1, 1), (1, 1), 1),
    (2, 64, 6, 10, 24, 1, 1, (1, 1), (0, 0), 1),
    (2, 128, 5, 9, 64, 1, 1, (1, 1), (0, 0), 1),
    # few output tiles and a long reduction: the reduction is split over several blocks
    (2, 256, 9, 9, 96, 3, 3, (2, 2), (0, 0), 1),
    (40, 520, 1, 1, 200, 1, 1, (1, 1), (0, 0), 1),
    # more strides
    (2, 64, 8, 8, 128, 1, 1, (2, 2), (0, 0), 1),       # 1x1 stride 2: most input pixels receive no gradient
    (1, 16, 9, 8, 24, 1, 1, (2, 2), (1, 1), 1),        # ... odd height, padding: the pixels with taps are the odd ones
    (1, 16, 9, 7, 24, 1, 1, (2, 2), (1, 1), 1),        # ... odd row length
    (2, 8, 6, 10, 16, 1, 1, (3, 2), (0, 0), 1),
    (1, 8, 5, 12, 8, 3, 1, (1, 2), (1, 0), 1),         # stride along the row only, three taps along the column
    (2, 200, 8, 8, 520, 1, 1, (2, 2), (0, 0), 1),      # ... with a split reduction
    (2, 40, 9, 10, 72, 3, 3, (2, 2), (1, 1), 1),
    (1, 16, 13, 11, 24, 5, 3, (3, 2), (2, 1), 1),
    (1, 16, 7, 7, 16, 2, 2, (3, 3), (0, 0), 1),        # stride larger than the filter: pixels no tap reaches
    # 3x3 under stride 2: backward-weight walks image rows with two input positions per gradient position
    (3, 40, 23, 12, 72, 3, 3, (2, 2), (0, 2), 1),      # no padding along H, 2 along W; even row length
    (5, 130, 21, 11, 70, 3, 3, (2, 2), (2, 0), 1),     # 60 gradient rows: two chunks of 32 lines; odd row length
    (2, 16, 8, 35, 16, 3, 3, (2, 2), (1, 1), 1),       # 18 steps per line: exactly three ring stages
    # strided backward-data split into residue classes of the pixels: rows of at least 24 pixels, or a
    # reduction of at least 2048 bytes per pixel
    (1, 16, 9, 26, 24, 3, 3, (2, 2), (1, 1), 1),
    (2, 70, 7, 37, 8, 5, 3, (3, 2), (2, 1), 1),        # 3 x 2 classes of unequal size, two row tiles
    (1, 8, 30, 30, 16, 2, 2, (2, 2), (0, 0), 1),       # every class has exactly one tap
    (1, 12, 5, 50, 20, 3, 5, (1, 2), (1, 2), 1),       # strided along the row only
    (1, 8, 9, 9, 240, 3, 3, (2, 2), (1, 1), 1),
    (2, 130, 9, 9, 240, 3, 3, (2, 2), (1, 1), 1),      # ... with the reduction of each class split over blocks
    (1, 40, 33, 6, 130, 4, 3, (3, 1), (0, 1), 1),      # strided along the column only, stride 3 on a 4-tap filter
    # stride 2 with at most 4 input channels: backward-weight runs on the space-to-depth image
    (2, 3, 12, 10, 8, 7, 7, (2, 2), (3, 3), 1),
    (17, 3, 16, 16, 70, 7, 7, (2, 2), (3, 3), 1),      # more than one image group and filter tile
    (1, 4, 8, 8, 5, 3, 3, (2, 2), (1, 1), 1),
    (2, 2, 6, 8, 4, 2, 2, (2, 2), (0, 0), 1),
    (1, 1, 10, 12, 3, 5, 3, (2, 2), (2, 0), 1),
    (3, 3, 8, 8, 6, 4, 6, (2, 2), (1, 2), 1),          # even filter, even and odd padding
    (2, 3, 9, 8, 6, 3, 3, (2, 2), (1, 1), 1),          # odd image height: the last block row is half empty
    (1, 3, 11, 13, 5, 3, 3, (2, 2), (0, 0), 1),        # odd both ways, no padding
    (2, 2, 7, 9, 4, 5, 5, (2, 2), (2, 2), 1),
]


@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_conv_three_passes_bit_exact(shape):
    N, C, H, W, K, R, S, st, pd, g = shape
    od = oracle.make_desc(N, C, H, W, K, R, S, st, pd, g)
    gd = B.make_desc(N, C, H, W, K, R, S, st, pd, g)
    P, Q = oracle.out_hw(od)
    r = np.random.RandomState(abs(hash(shape)) % 2 ** 31)
    x = r.randint(-127, 128, size=(N, C, H, W)).astype(np.int8)
    w = r.randint(-127, 128, size=(K, C // g, R, S)).astype(np.int8)
    dy = r.randint(-127, 128, size=(N, K, P, Q)).astype(np.int8)
    dwise = g != 1
    xq = dev(x.reshape(-1) if dwise else pack_act(x))
    dyq = dev(dy.reshape(-1) if dwise else pack_act(dy))
    wq = dev(w.reshape(-1) if dwise else pack_wgt(w))
    sx, sw, sdy = (dev(np.array([v], np.float32)) for v in (0.0123, 3.3e-3, 7.7e-6))
    ws = torch.empty(max(256, *(B.int8t_workspace_bytes(op, gd) for op in
                                (B.OP_CONV_FWD, B.OP_CONV_BWD_DATA, B.OP_CONV_BWD_WEIGHT))),
                     dtype=torch.uint8, device=DEV)

    def run(fn, a, sa, b, sb, shape_out):
        out = torch.full(shape_out, float("nan"), dtype=torch.float32, device=DEV)
        acc = torch.full(shape_out, -12345, dtype=torch.int32, device=DEV)
        fn(gd, a, sa, b, sb, out, acc, ws)
        torch.cuda.synchronize()
        return out.cpu().numpy(), acc.cpu().numpy()

    for name, got, want64, s1, s2 in (
        ("fwd", run(B.int8t_conv_fwd, xq, sx, wq, sw, (N, K, P, Q)), oracle.conv_fwd(od, x, w), 0.0123, 3.3e-3),
        ("bwd_data", run(B.int8t_conv_bwd_data, dyq, sdy, wq, sw, (N, C, H, W)),
         oracle.conv_bwd_data(od, dy, w), 7.7e-6, 3.3e-3),
        ("bwd_weight", run(B.int8t_conv_bwd_weight, xq, sx, dyq, sdy, (K, C // g, R, S)),
         oracle.conv_bwd_weight(od, x, dy), 0.0123, 7.7e-6),
    ):
        out, acc = got
        want32, ov = oracle.wrap32(want64)
        assert ov == 0
        assert np.array_equal(acc, want32), name
        ref = oracle.dequant(want32, np.float32(s1), np.float32(s2))
        assert np.all(np.abs(out - ref) <= REL_TOL * np.abs(ref)), name


def test_conv_three_passes_random_shapes():
    """120 seeded random small layers (filters 1..7, strides 1..3, any padding below the filter, dense
    and depthwise, ragged channel counts): accumulators and results of all three passes, bit for bit."""
    r = np.random.RandomState(2)
    one = dev(np.array([1.0], np.float32))
    done = 0
    while done < 120:
        dwise = r.rand() < 0.3
        R, S = int(r.choice([1, 2, 3, 5, 7])), int(r.choice([1, 2, 3, 5, 7]))
        if r.rand() < 0.5:
            S = R
        sh, sw = int(r.choice([1, 1, 2, 2, 3])), int(r.choice([1, 1, 2, 2, 3]))
        if r.rand() < 0.6:
            sw = sh
        ph, pw = int(r.randint(0, R)), int(r.randint(0, S))
        H, W = int(r.randint(R, 40)), int(r.randint(S, 40))
        if r.rand() < 0.3:
            W = (W + 3) & ~3
        N = int(r.randint(1, 5))
        if dwise:
            C = K = g = int(r.randint(2, 20))
        else:
            C, K, g = int(r.choice([1, 3, 4, 16, 24, 40, 70, 130])), int(r.choice([4, 16, 24, 64, 72, 130, 250])), 1
        od = oracle.make_desc(N, C, H, W, K, R, S, (sh, sw), (ph, pw), g)
        P, Q = oracle.out_hw(od)
        if P < 1 or Q < 1:
            continue
        done += 1
        shape = (N, C, H, W, K, R, S, (sh, sw), (ph, pw), g)
        gd = B.make_desc(*shape)
        x = r.randint(-127, 128, size=(N, C, H, W)).astype(np.int8)
        w = r.randint(-127, 128, size=(K, C // g, R, S)).astype(np.int8)
        dy = r.randint(-127, 128, size=(N, K, P, Q)).astype(np.int8)
        xq = dev(x.reshape(-1) if dwise else pack_act(x))
        dyq = dev(dy.reshape(-1) if dwise else pack_act(dy))
        wq = dev(w.reshape(-1) if dwise else pack_wgt(w))
        ws = torch.empty(max(256, *(B.int8t_workspace_bytes(op, gd) for op in
                                    (B.OP_CONV_FWD, B.OP_CONV_BWD_DATA, B.OP_CONV_BWD_WEIGHT))),
                         dtype=torch.uint8, device=DEV)
        for name, fn, a, b, so, want in (
            ("fwd", B.int8t_conv_fwd, xq, wq, (N, K, P, Q), oracle.conv_fwd(od, x, w)),
            ("bwd_data", B.int8t_conv_bwd_data, dyq, wq, (N, C, H, W), oracle.conv_bwd_data(od, dy, w)),
            ("bwd_weight", B.int8t_conv_bwd_weight, xq, dyq, (K, C // g, R, S), oracle.conv_bwd_weight(od, x, dy)),
        ):
            out = torch.full(so, float("nan"), dtype=torch.float32, device=DEV)
            acc = torch.full(so, -12345, dtype=torch.int32, device=DEV)
            fn(gd, a, one, b, one, out, acc, ws)
            torch.cuda.synchronize()
            want32, _ = oracle.wrap32(want)
            assert np.array_equal(acc.cpu().numpy(), want32), (name, shape)
            assert np.array_equal(out.cpu().numpy(), want32.astype(np.float32)), (name, shape)   # scales are 1


# Layers large enough for the 128-row and the 256 x 256 tiles of igemm_dma_kernel (forward / backward-data
# of every layer with more than 64 output rows run it; 256 x 256 from 192 such tiles up), plain, split by
# pixel classes and in the cell form; every accumulator and every fp32 result is compared.
# (N, C, H, W, K, R, S, stride, pad, groups), passes that must run the wide kernel
WIDE_SHAPES = [
    # forward and plain backward-data, 128-row tiles (192 rows: one full and one half row tile; ragged columns)
    ((4, 192, 95, 97, 192, 1, 3, (1, 1), (0, 1), 1), ("fwd", "bwd_data")),
    # ... a larger batch: at least 192 tiles of 256 x 256, which the plain passes then take
    ((6, 192, 95, 97, 192, 1, 3, (1, 1), (0, 1), 1), ("fwd", "bwd_data")),
    # backward-data by residue classes (3 x 3, stride 2: four classes with 4, 2, 2, 1 taps)
    ((2, 192, 127, 129, 128, 3, 3, (2, 2), (1, 1), 1), ("bwd_data",)),
    # ... a larger batch
    ((3, 192, 127, 129, 128, 3, 3, (2, 2), (1, 1), 1), ("bwd_data",)),
    # backward-data in the cell form (1 x 1, stride 2, even row length, odd height)
    ((32, 192, 63, 64, 512, 1, 1, (2, 2), (0, 0), 1), ("bwd_data",)),
    # ... a larger batch
    ((48, 192, 63, 64, 512, 1, 1, (2, 2), (0, 0), 1), ("bwd_data",)),
    # backward-data with the four pixel classes of stride 2 in one block (rows of at least 28 pixels, even length):
    # odd height, so that the last cell row is half empty
    ((2, 130, 57, 60, 64, 3, 3, (2, 2), (1, 1), 1), ("bwd_data",)),
]


@pytest.mark.parametrize("shape,wide_passes", WIDE_SHAPES)
def test_wide_tile_kernels_elementwise(shape, wide_passes):
    N, C, H, W, K, R, S, st, pd, g = shape
    od = oracle.make_desc(N, C, H, W, K, R, S, st, pd, g)
    gd = B.make_desc(N, C, H, W, K, R, S, st, pd, g)
    P, Q = oracle.out_hw(od)
    r = np.random.RandomState(abs(hash(shape)) % 2 ** 31)
    x = r.randint(-127, 128, size=(N, C, H, W)).astype(np.int8)
    w = r.randint(-127, 128, size=(K, C, R, S)).astype(np.int8)
    dy = r.randint(-127, 128, size=(N, K, P, Q)).astype(np.int8)
    xq, dyq, wq = dev(pack_act(x)), dev(pack_act(dy)), dev(pack_wgt(w))
    s1, s2 = np.float32(0.0123), np.float32(3.3e-3)
    sa, sb = dev(np.array([s1], np.float32)), dev(np.array([s2], np.float32))
    for name, fn, op, a, shape_out, want_fn, args in (
        ("fwd", B.int8t_conv_fwd, B.OP_CONV_FWD, xq, (N, K, P, Q), oracle.conv_fwd, (x, w)),
        ("bwd_data", B.int8t_conv_bwd_data, B.OP_CONV_BWD_DATA, dyq, (N, C, H, W), oracle.conv_bwd_data, (dy, w)),
    ):
        if name not in wide_passes:
            continue
        nws = B.int8t_workspace_bytes(op, gd)
        ws = torch.empty(nws, dtype=torch.uint8, device=DEV) if nws else None
        out = torch.full(shape_out, float("nan"), dtype=torch.float32, device=DEV)
        acc = torch.full(shape_out, -12345, dtype=torch.int32, device=DEV)
        B.int8t_profile_start(None)
        fn(gd, a, sa, wq, sb, out, acc, ws)
        torch.cuda.synchronize()
        ran = B.int8t_profile_stop()
        assert list(ran) == ["igemm_dma_kernel"], (name, ran)       # the kernel under test, and nothing else
        want32, ov = oracle.wrap32(want_fn(od, *args))
        assert ov == 0
        assert np.array_equal(acc.cpu().numpy(), want32), name
        ref = oracle.dequant(want32, s1, s2)
        assert np.all(np.abs(out.cpu().numpy() - ref) <= REL_TOL * np.abs(ref)), name


@pytest.mark.parametrize("shape", [
    (2, 256, 9, 9, 96, 3, 3, (1, 1), (1, 1), 1),       # split reduction in both passes
    (2, 3, 12, 10, 8, 7, 7, (2, 2), (3, 3), 1),        # forward pass on the space-to-depth codes
])
def test_conv_without_optional_workspace(shape):
    # forward / backward-data take their scratch as a hint: without it the result is the same
    N, C, H, W, K, R, S, st, pd, g = shape
    gd = B.make_desc(N, C, H, W, K, R, S, st, pd, g)
    assert B.int8t_workspace_bytes(B.OP_CONV_FWD, gd) > 0
    P, Q = oracle.out_hw(oracle.make_desc(N, C, H, W, K, R, S, st, pd, g))
    r = np.random.RandomState(7)
    x = r.randint(-127, 128, size=(N, C, H, W)).astype(np.int8)
    w = r.randint(-127, 128, size=(K, C, R, S)).astype(np.int8)
    dy = r.randint(-127, 128, size=(N, K, P, Q)).astype(np.int8)
    xq, dyq, wq = dev(pack_act(x)), dev(pack_act(dy)), dev(pack_wgt(w))
    one = dev(np.array([1.0], np.float32))
    for fn, op, a, shape_out in ((B.int8t_conv_fwd, B.OP_CONV_FWD, xq, (N, K, P, Q)),
                                 (B.int8t_conv_bwd_data, B.OP_CONV_BWD_DATA, dyq, (N, C, H, W))):
        res = []
        for nbytes in (B.int8t_workspace_bytes(op, gd), 0, 256):
            ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV) if nbytes else None
            out = torch.full(shape_out, float("nan"), dtype=torch.float32, device=DEV)
            acc = torch.full(shape_out, -12345, dtype=torch.int32, device=DEV)
            fn(gd, a, one, wq, one, out, acc, ws)
            torch.cuda.synchronize()
            res.append((out.cpu().numpy(), acc.cpu().numpy()))
        for o, a_ in res[1:]:
            assert np.array_equal(a_, res[0][1]) and np.array_equal(o, res[0][0])


def test_bwd_weight_int32_wrap():
    # 133145 products of 127*127 exceed 2^31: the accumulator wraps to a known value
    N, P, Q = 5, 31, 859
    od = oracle.make_desc(N, 1, P, Q, 1, 1, 1)
    gd = B.make_desc(N, 1, P, Q, 1, 1, 1)
    x = np.full((N, 1, P, Q), 127, np.int8)
    ws = torch.empty(max(256, B.int8t_workspace_bytes(B.OP_CONV_BWD_WEIGHT, gd)), dtype=torch.uint8, device=DEV)
    out = torch.zeros((1, 1, 1, 1), dtype=torch.float32, device=DEV)
    acc = torch.zeros((1, 1, 1, 1), dtype=torch.int32, device=DEV)
    one = dev(np.array([1.0], np.float32))
    xq = dev(pack_act(x))
    B.int8t_conv_bwd_weight(gd, xq, one, xq, one, out, acc, ws)
    torch.cuda.synchronize()
    want32, ov = oracle.wrap32(oracle.conv_bwd_weight(od, x, x))
    assert ov == 1 and acc.item() == want32.item() == -2147471591
    assert out.item() == np.float32(-2147471591)


def run_layer(cfg, li, keep_acc=True):
    L, x, w, dy = inputs.make_layer_inputs(cfg, li)
    st = LayerStep(L, n_cand=32, keep_acc=keep_acc)
    st.upload(x, w, dy, inputs.default_ratios(32))
    st.run(seed=0)
    torch.cuda.synchronize()
    return L, x, w, dy, st


def test_config0_full_step_elementwise():
    L, x, w, dy, st = run_layer(0, 0)
    od = oracle.make_desc(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad, L.groups)
    xq, sx = oracle.quantize(x)
    wq, sw = oracle.quantize(w)
    o = oracle.dsgc(dy.reshape(-1), inputs.default_ratios(32), mode=STO, seed=0)
    assert np.all(np.abs(st.dev_all.cpu().numpy() - o["dev"]) < DEV_TOL)
    assert st.clip.item() == o["clip"]
    dyq, sdy = oracle.quantize(dy, c=o["clip"], mode=STO, seed=0)
    assert np.array_equal(st.codes_x(), xq) and st.sx.item() == sx
    a, b = st.codes_w()
    assert np.array_equal(a, wq) and np.array_equal(b, wq) and st.sw.item() == sw
    assert np.array_equal(st.codes_dy(), dyq) and st.sdy.item() == sdy
    assert abs(st.dev_final.item() - oracle.deviation(dy, dyq, sdy)) < DEV_TOL
    assert abs(st.dev_final.item() - st.dev_search.item()) < DEV_TOL
    for got, acc, want64, s1, s2 in (
        (st.y, st.y_acc, oracle.conv_fwd(od, xq, wq), sx, sw),
        (st.dx, st.dx_acc, oracle.conv_bwd_data(od, dyq, wq), sdy, sw),
        (st.dw, st.dw_acc, oracle.conv_bwd_weight(od, xq, dyq), sx, sdy),
    ):
        want32, ov = oracle.wrap32(want64)
        assert ov == 0 and np.array_equal(acc.cpu().numpy(), want32)
        ref = oracle.dequant(want32, s1, s2)
        assert np.all(np.abs(got.cpu().numpy() - ref) <= REL_TOL * np.abs(ref))
    phi = B.int8t_dclr_scale(st.dev_final.item())
    assert phi == oracle.dclr(st.dev_final.item())


FULL_LAYERS = [(1, 0), (2, 0), (2, 1), (2, 2), (3, 0), (3, 1), (3, 2), (4, 0), (4, 1), (4, 2), (5, 0),
               (6, 0), (6, 1), (6, 2)]


@pytest.mark.parametrize("cfg,li", FULL_LAYERS)
def test_full_size_layers(cfg, li):
    """Benchmark-size layers in the benchmark's launch configuration, everything compared in full:
    the three code tensors, the clip search (every candidate's deviation), and every int32
    accumulator and fp32 result of the three convolutions against the oracle's whole-tensor sums."""
    L, x, w, dy, st = run_layer(cfg, li)
    od = oracle.make_desc(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad, L.groups)
    xq, sx = oracle.quantize(x)
    wq, sw = oracle.quantize(w)
    assert np.array_equal(st.codes_x(), xq) and st.sx.item() == sx
    a, b = st.codes_w()
    assert np.array_equal(a, wq) and st.sw.item() == sw and (b is None or np.array_equal(b, wq))
    o = oracle.dsgc(dy.reshape(-1), inputs.default_ratios(32), mode=STO, seed=0)
    assert np.all(np.abs(st.dev_all.cpu().numpy() - o["dev"]) < DEV_TOL)
    clip = np.float32(st.clip.item())
    j = int(np.argmin(np.abs(o["clips"] - clip)))
    assert clip == o["clips"][j] and o["dev"][j] - o["deviation"] <= 2 * DEV_TOL
    dyq, sdy = oracle.quantize(dy, c=clip, mode=STO, seed=0)
    assert np.array_equal(st.codes_dy(), dyq) and st.sdy.item() == sdy
    assert abs(st.dev_final.item() - o["dev"][j]) < DEV_TOL

    for name, acc, out, want64, s1, s2 in (
        ("fwd", st.y_acc, st.y, oracle.conv_fwd(od, xq, wq), sx, sw),
        ("bwd_data", st.dx_acc, st.dx, oracle.conv_bwd_data(od, dyq, wq), sdy, sw),
        ("bwd_weight", st.dw_acc, st.dw, oracle.conv_bwd_weight(od, xq, dyq), sx, sdy),
    ):
        want32, ov = oracle.wrap32(want64)
        assert ov == 0, name                       # the benchmark's distributions stay inside int32
        got = acc.cpu().numpy()
        assert np.array_equal(got, want32), (name, int((got != want32).sum()))
        ref = oracle.dequant(want32, s1, s2)
        assert np.all(np.abs(out.cpu().numpy() - ref) <= REL_TOL * np.abs(ref)), name


@pytest.mark.parametrize("cfg,li", [(0, 0), (1, 0), (3, 1)])
def test_two_stream_step_equals_one_stream_step(cfg, li):
    """Every two-stream schedule of the step (the a / W chain and the forward pass beside the search,
    backward-weight beside the other convolutions, both) writes exactly what the one-stream step writes
    (several steps in a row, so that the streams' hand-overs are exercised)."""
    L, x, w, dy = inputs.make_layer_inputs(cfg, li)
    outs = []
    for overlap in (False, True, 2, 3, 4):
        st = LayerStep(L, n_cand=32, keep_acc=True)
        st.upload(x, w, dy, inputs.default_ratios(32))
        for seed in (5, 6, 7):
            st.run(seed=seed, overlap=overlap)
        torch.cuda.synchronize()
        outs.append([t.clone() for t in (st.xq, st.wq, st.dyq, st.sx, st.sw, st.sdy, st.clip, st.dev_search,
                                          st.y, st.dx, st.dw, st.y_acc, st.dx_acc, st.dw_acc)])
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert torch.equal(a, b)


@pytest.mark.parametrize("cfg,li", [(0, 0), (3, 1), (5, 0)])
def test_step_that_keeps_the_clip_equals_step_that_searches(cfg, li):
    """Periodic Update: a step with search=False reuses the clip value in device memory (and quantizes
    a, W and g_z in one batched call); with the same seed it must write what the searching step wrote."""
    L, x, w, dy = inputs.make_layer_inputs(cfg, li)
    st = LayerStep(L, n_cand=32, requantize_deviation=False)
    st.upload(x, w, dy, inputs.default_ratios(32))
    st.run(seed=3, search=True)
    torch.cuda.synchronize()
    want = [t.clone() for t in (st.xq, st.wq, st.dyq, st.sx, st.sw, st.sdy, st.y, st.dx, st.dw)]
    for t in (st.xq, st.wq, st.dyq, st.y, st.dx, st.dw):
        t.zero_()
    st.run(seed=3, search=False)
    torch.cuda.synchronize()
    for a, b in zip(want, (st.xq, st.wq, st.dyq, st.sx, st.sw, st.sdy, st.y, st.dx, st.dw)):
        assert torch.equal(a, b)


@pytest.mark.parametrize("cfg,li", [(0, 0), (2, 1), (3, 1)])
def test_forked_step_that_keeps_the_clip_equals_one_stream_step(cfg, li):
    """A step that keeps the clip with backward-weight on the second stream writes what the one-stream step
    writes (several steps in a row with changing seeds, so that each step's hand-overs are exercised)."""
    L, x, w, dy = inputs.make_layer_inputs(cfg, li)
    outs = []
    # (schedule, deviation of the final codes asked for: the step then quantizes g_z in a call of its own)
    for overlap, requant in ((False, False), (True, False), (False, True), (2, True), (3, True), (4, True)):
        st = LayerStep(L, n_cand=32, keep_acc=True, requantize_deviation=requant)
        st.upload(x, w, dy, inputs.default_ratios(32))
        st.run(seed=5, overlap=False)
        for t in (st.xq, st.wq, st.dyq, st.y, st.dx, st.dw):
            t.zero_()
        for seed in (6, 7, 8):
            st.run(seed=seed, search=False, overlap=overlap)
        torch.cuda.synchronize()
        outs.append([t.clone() for t in (st.xq, st.wq, st.dyq, st.sx, st.sw, st.sdy, st.clip,
                                          st.y, st.dx, st.dw, st.y_acc, st.dx_acc, st.dw_acc)])
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert torch.equal(a, b)


def test_tuned_schedule_writes_the_same_tensors():
    L, x, w, dy = inputs.make_layer_inputs(1, 0)
    st = LayerStep(L, n_cand=32, requantize_deviation=False)
    st.upload(x, w, dy, inputs.default_ratios(32))
    st.run(seed=4, overlap=False)
    torch.cuda.synchronize()
    want = [t.clone() for t in (st.dyq, st.y, st.dx, st.dw, st.clip)]
    choice = st.tune(steps=5)
    assert choice in (0, 1, 2, 3, 4)
    st.run(seed=4)                      # overlap=None: the tuned schedule
    torch.cuda.synchronize()
    for a, b in zip(want, (st.dyq, st.y, st.dx, st.dw, st.clip)):
        assert torch.equal(a, b)
    for t in (st.dyq, st.y, st.dx, st.dw):
        t.zero_()
    st.run(seed=4, search=False)        # ... and the tuned schedule of a step that keeps the clip
    torch.cuda.synchronize()
    for a, b in zip(want, (st.dyq, st.y, st.dx, st.dw, st.clip)):
        assert torch.equal(a, b)


@pytest.mark.parametrize("shape", [(2, 24, 9, 9, 144), (3, 144, 7, 7, 24), (2, 70, 5, 6, 130), (33, 200, 1, 1, 70), (2, 16, 16, 16, 300)])
def test_fused_quantize_conv_equals_separate_calls_and_oracle(shape):
    """int8t_conv_fwd_fused (Eq.1 inside the forward pass of a 1x1 stride-1 layer) writes the codes, the
    scale, the accumulators and the results of int8t_quantize + int8t_conv_fwd, which are the oracle's."""
    N, C, H, W, K = shape
    r = np.random.RandomState(N * 100 + C)
    x = (r.standard_normal((N, C, H, W)) * 1.7).astype(np.float32)
    x[0, 0, 0, 0] = np.nan if C > 20 else x[0, 0, 0, 0]
    w = r.randint(-127, 128, size=(K, C, 1, 1)).astype(np.int8)
    gd = B.make_desc(N, C, H, W, K, 1, 1)
    od = oracle.make_desc(N, C, H, W, K, 1, 1)
    wq, sw = dev(pack_wgt(w)), dev(np.array([3.3e-3], np.float32))
    xd = dev(x)
    ws = torch.empty(4096, dtype=torch.uint8, device=DEV)
    for clip in (None, 2.5):
        cd = None if clip is None else dev(np.array([clip], np.float32))
        for want_codes in (True, False):
            y = torch.full((N, K, H, W), float("nan"), dtype=torch.float32, device=DEV)
            acc = torch.full((N, K, H, W), -12345, dtype=torch.int32, device=DEV)
            xq = torch.full((B.int8t_code_bytes(x.shape, B.ACT),), 77, dtype=torch.int8, device=DEV) if want_codes else None
            sx = torch.zeros(1, dtype=torch.float32, device=DEV)
            B.int8t_conv_fwd_fused(gd, xd, cd, wq, sw, y, acc, xq, sx, ws)
            torch.cuda.synchronize()
            qo, so = oracle.quantize(x, c=clip)
            assert sx.item() == so
            if want_codes:
                q2, s2, _ = gpu_quantize(x, B.ACT, clip)
                assert np.array_equal(xq.cpu().numpy(), q2) and s2 == so            # incl. zero channel padding
                assert np.array_equal(unpack_act(xq.cpu().numpy(), x.shape, False), qo)
            want32, ov = oracle.wrap32(oracle.conv_fwd(od, qo, w))
            assert ov == 0 and np.array_equal(acc.cpu().numpy(), want32)
            ref = oracle.dequant(want32, so, np.float32(3.3e-3))
            assert np.all(np.abs(y.cpu().numpy() - ref) <= REL_TOL * np.abs(ref))
    with pytest.raises(B.Int8tError) as e:
        B.int8t_conv_fwd_fused(B.make_desc(N, C, H + 2, W + 2, K, 3, 3), xd, None, wq, sw, y, None, None, sx, ws)
    assert e.value.status == 2


def test_step_with_fused_forward_equals_plain_step():
    L, x, w, dy = inputs.make_layer_inputs(3, 2)
    outs = []
    for fused in (False, True):
        for overlap in (False, True, 2, 3, 4):
            st = LayerStep(L, n_cand=32, keep_acc=True, fused_fwd=fused)
            st.upload(x, w, dy, inputs.default_ratios(32))
            st.wq.zero_()                  # (the alignment gap between the two weight layouts is never written)
            for seed in (5, 6):
                st.run(seed=seed, overlap=overlap)
            torch.cuda.synchronize()
            outs.append([t.clone() for t in (st.xq, st.wq, st.dyq, st.sx, st.sw, st.sdy, st.y, st.dx, st.dw, st.y_acc, st.dw_acc)])
    names = ("xq", "wq", "dyq", "sx", "sw", "sdy", "y", "dx", "dw", "y_acc", "dw_acc")
    for k, other in enumerate(outs[1:]):
        for name, a, b in zip(names, outs[0], other):
            assert torch.equal(a, b), (k + 1, name, int((a != b).sum()))


def test_every_kernel_variant_is_exact():
    """Per-layer kernel choice: every variant int8t_conv_variant_ok() admits for a pass of a layer --
    i.e. everything a tuner may select -- writes the oracle's accumulators and results, on small layers
    with ragged channels, several taps, strides and padding (each variant also runs layers it would never
    be chosen for).  The selection is restored to the library's own choice afterwards."""
    shapes = [(2, 16, 16, 16, 32, 3, 3, (1, 1), (1, 1), 1), (3, 64, 14, 14, 130, 3, 3, (1, 1), (1, 1), 1),
              (2, 70, 9, 11, 40, 1, 7, (1, 1), (0, 3), 1), (2, 256, 9, 9, 96, 3, 3, (2, 2), (0, 0), 1),
              (2, 24, 9, 9, 144, 1, 1, (1, 1), (0, 0), 1), (1, 40, 33, 6, 130, 4, 3, (3, 1), (0, 1), 1),
              (2, 64, 8, 8, 128, 1, 1, (2, 2), (0, 0), 1), (40, 520, 1, 1, 200, 1, 1, (1, 1), (0, 0), 1),
              (2, 3, 12, 10, 8, 7, 7, (2, 2), (3, 3), 1), (17, 130, 7, 37, 72, 5, 3, (1, 2), (2, 1), 1),
              # stride 1, several taps; column tiles that span image borders
              (3, 64, 14, 14, 128, 3, 3, (1, 1), (1, 1), 1), (2, 128, 17, 17, 192, 1, 7, (1, 1), (0, 3), 1),
              (2, 64, 17, 17, 64, 7, 1, (1, 1), (3, 0), 1), (5, 64, 9, 11, 64, 3, 3, (1, 1), (0, 0), 1),
              (2, 64, 8, 8, 64, 2, 2, (1, 1), (1, 1), 1), (3, 192, 6, 7, 64, 3, 5, (1, 1), (1, 0), 1),
              (40, 64, 5, 5, 64, 3, 3, (1, 1), (1, 1), 1),        # column tiles that span many small images
              # backward-weight on image lines: ragged channel tiles, padding beyond the taps' reach, 7 taps
              # along H on few lines, 1x1 on 128 x 128 tiles with ragged edges
              (2, 40, 9, 13, 72, 3, 3, (1, 1), (1, 1), 1), (2, 64, 8, 8, 64, 3, 3, (1, 1), (2, 2), 1),
              (2, 48, 6, 20, 80, 7, 1, (1, 1), (3, 0), 1), (3, 130, 10, 6, 200, 1, 1, (1, 1), (0, 0), 1),
              (1, 256, 3, 37, 130, 1, 7, (1, 1), (0, 3), 1),
              # stride 2 x 2: backward-data on 2 x 2 cells with all four pixel classes in one block -- odd and even
              # images (the last cell row / column half empty), 5- and 2-tap filters, ragged rows, several column tiles
              (2, 40, 9, 10, 72, 3, 3, (2, 2), (1, 1), 1), (1, 16, 11, 13, 24, 5, 3, (2, 2), (2, 1), 1),
              (2, 130, 8, 8, 70, 2, 2, (2, 2), (0, 0), 1), (3, 200, 17, 17, 48, 3, 3, (2, 2), (0, 0), 1),
              (5, 24, 14, 15, 130, 3, 5, (2, 2), (1, 2), 1)]
    one = dev(np.array([1.0], np.float32))
    seen = set()
    for shape in shapes:
        N, C, H, W, K, R, S, st, pd, g = shape
        od = oracle.make_desc(*shape)
        gd = B.make_desc(*shape)
        P, Q = oracle.out_hw(od)
        r = np.random.RandomState(abs(hash(shape)) % 2 ** 31)
        x = r.randint(-127, 128, size=(N, C, H, W)).astype(np.int8)
        w = r.randint(-127, 128, size=(K, C, R, S)).astype(np.int8)
        dy = r.randint(-127, 128, size=(N, K, P, Q)).astype(np.int8)
        xq, dyq, wq = dev(pack_act(x)), dev(pack_act(dy)), dev(pack_wgt(w))
        for name, fn, op, a, b, so, want in (
            ("fwd", B.int8t_conv_fwd, B.OP_CONV_FWD, xq, wq, (N, K, P, Q), oracle.conv_fwd(od, x, w)),
            ("bwd_data", B.int8t_conv_bwd_data, B.OP_CONV_BWD_DATA, dyq, wq, (N, C, H, W), oracle.conv_bwd_data(od, dy, w)),
            ("bwd_weight", B.int8t_conv_bwd_weight, B.OP_CONV_BWD_WEIGHT, xq, dyq, (K, C, R, S), oracle.conv_bwd_weight(od, x, dy)),
        ):
            want32, _ = oracle.wrap32(want)
            try:
                for v in range(len(B.VARIANT_NAMES)):
                    if not B.int8t_conv_variant_ok(op, gd, v):
                        with pytest.raises(B.Int8tError):
                            B.int8t_conv_select_variant(op, gd, v)
                        continue
                    B.int8t_conv_select_variant(op, gd, v)
                    assert B.int8t_conv_selected_variant(op, gd) == v
                    seen.add((name, v))
                    ws = torch.empty(max(256, B.int8t_workspace_bytes(op, gd)), dtype=torch.uint8, device=DEV)
                    out = torch.full(so, float("nan"), dtype=torch.float32, device=DEV)
                    acc = torch.full(so, -12345, dtype=torch.int32, device=DEV)
                    fn(gd, a, one, b, one, out, acc, ws)
                    torch.cuda.synchronize()
                    assert np.array_equal(acc.cpu().numpy(), want32), (name, B.VARIANT_NAMES[v], shape)
                    assert np.array_equal(out.cpu().numpy(), want32.astype(np.float32)), (name, B.VARIANT_NAMES[v], shape)
            finally:
                B.int8t_conv_select_variant(op, gd, B.VARIANT_AUTO)
    # every variant ran at least once in each pass it exists for
    for v in (B.VARIANT_BAND, B.VARIANT_TILE, B.VARIANT_TILE_SPLIT, B.VARIANT_WIDE128, B.VARIANT_WIDE256, B.VARIANT_WIDE_SQ128,
              B.VARIANT_WIDE_SQ128_DEEP, B.VARIANT_WIDE_128X64):
        assert ("fwd", v) in seen and ("bwd_data", v) in seen, B.VARIANT_NAMES[v]
    assert ("bwd_data", B.VARIANT_WIDE_CELLS) in seen and ("fwd", B.VARIANT_WIDE_CELLS) not in seen
    for v in (B.VARIANT_WGRAD_FEWER, B.VARIANT_WGRAD_MORE, B.VARIANT_WGRAD_IMAGES, B.VARIANT_WGRAD_LINES):
        assert ("bwd_weight", v) in seen, B.VARIANT_NAMES[v]


def test_tuned_kernels_write_the_same_tensors():
    L, x, w, dy = inputs.make_layer_inputs(2, 1)
    st = LayerStep(L, n_cand=32, requantize_deviation=False, keep_acc=True)
    st.upload(x, w, dy, inputs.default_ratios(32))
    st.run(seed=4, overlap=False)
    torch.cuda.synchronize()
    want = [t.clone() for t in (st.y, st.dx, st.dw, st.y_acc, st.dx_acc, st.dw_acc)]
    try:
        choice = st.tune_kernels(reps=5)
        assert set(choice) == {"fwd", "bwd_data", "bwd_weight"}
        for t in (st.y, st.dx, st.dw):
            t.zero_()
        st.run(seed=4, overlap=False)
        torch.cuda.synchronize()
        for a, b in zip(want, (st.y, st.dx, st.dw, st.y_acc, st.dx_acc, st.dw_acc)):
            assert torch.equal(a, b)
    finally:
        for op in (B.OP_CONV_FWD, B.OP_CONV_BWD_DATA, B.OP_CONV_BWD_WEIGHT):
            B.int8t_conv_select_variant(op, st.desc, B.VARIANT_AUTO)


def test_same_seed_same_codes_different_seed_differs():
    L, x, w, dy = inputs.make_layer_inputs(0, 0)
    a, _, _ = gpu_quantize(dy, B.ACT, 0.01, STO, seed=42)
    b, _, _ = gpu_quantize(dy, B.ACT, 0.01, STO, seed=42)
    c, _, _ = gpu_quantize(dy, B.ACT, 0.01, STO, seed=43)
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    # layout independence: planar and channels-last layouts hold the same logical codes
    p, _, _ = gpu_quantize(dy, B.ACT_PLANAR, 0.01, STO, seed=42)
    assert np.array_equal(unpack_act(a, dy.shape, False), p.reshape(dy.shape))


def test_error_paths_on_device():
    x = torch.zeros(64, dtype=torch.float32, device=DEV)
    q = torch.zeros(1024, dtype=torch.int8, device=DEV)
    s = torch.zeros(1, dtype=torch.float32, device=DEV)
    with pytest.raises(B.Int8tError) as e:
        B.int8t_quantize(x, (1, 4, 4, 4), B.ACT, None, RTN, 0, q, s, None, torch.zeros(16, dtype=torch.uint8, device=DEV))
    assert e.value.status == 4
    with pytest.raises(B.Int8tError) as e:
        B.int8t_quantize(x, (1, 4, 4, 4), 9, None, RTN, 0, q, s, None, None)
    assert e.value.status == 3
