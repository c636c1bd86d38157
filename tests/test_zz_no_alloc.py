"""int8t_dsgc_clip_static -- the clip search for callers that cannot allocate -- against
int8t_dsgc_clip with caller scratch: clip value, winning deviation and every candidate's deviation
must be identical (both run the same kernels; the sums are exact integers plus fixed-order fp64), on
two calls in a row that share the GPU's static scratch, the second on a smaller input, and against
the oracle's brute-force search to the parity bar (1e-9)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

import oracle  # noqa: E402
from paper_1912_12607_amd import binding as B  # noqa: E402
from paper_1912_12607_amd import inputs  # noqa: E402

DEV = torch.device("cuda:0")


def search(g, ratios, seed, static):
    gd = torch.from_numpy(g).to(DEV)
    rd = torch.from_numpy(np.asarray(ratios, np.float32)).to(DEV)
    J = len(ratios)
    clip = torch.full((1,), -1.0, dtype=torch.float32, device=DEV)
    d = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    da = torch.full((J,), -1.0, dtype=torch.float64, device=DEV)
    if static:
        B.int8t_dsgc_clip_static(gd, g.size, rd, J, B.ROUND_STOCHASTIC, seed, clip, d, da)
    else:
        ws = torch.empty(B.int8t_workspace_bytes(B.OP_DSGC, None, g.size, J), dtype=torch.uint8, device=DEV)
        B.int8t_dsgc_clip(gd, g.size, rd, J, B.ROUND_STOCHASTIC, seed, clip, d, da, ws)
    torch.cuda.synchronize()
    return np.float32(clip.item()), d.item(), da.cpu().numpy()


def test_static_scratch_variant_equals_the_caller_scratch_variant():
    r = np.random.RandomState(8)
    ratios = inputs.default_ratios(32)
    big = (r.standard_t(3, size=1_500_003) * 1e-3).astype(np.float32)     # ragged tail, every block busy
    big[r.choice(big.size, 150, replace=False)] *= 100
    small = (r.standard_t(3, size=70_001) * 1e-4).astype(np.float32)
    results = []
    for g, seed in ((big, 11), (small, 12)):          # two calls in a row on the same static scratch
        results.append((g, seed, search(g, ratios, seed, static=True)))
    for g, seed, (clip_s, d_s, da_s) in results:
        clip_w, d_w, da_w = search(g, ratios, seed, static=False)
        assert clip_s == clip_w and d_s == d_w and np.array_equal(da_s, da_w)
        o = oracle.dsgc(g, ratios, mode=oracle.ROUND_STOCHASTIC, seed=seed)
        assert np.all(np.abs(da_s - o["dev"]) < 1e-9)
        j = int(np.argmin(np.abs(o["clips"] - clip_s)))
        assert clip_s == o["clips"][j] and o["dev"][j] - o["deviation"] <= 2e-9 and abs(d_s - o["dev"][j]) < 1e-9


def test_static_variant_limits_and_argument_errors():
    g = torch.zeros(64, dtype=torch.float32, device=DEV)
    rd = torch.ones(80, dtype=torch.float32, device=DEV)
    clip = torch.zeros(1, dtype=torch.float32, device=DEV)
    d = torch.zeros(1, dtype=torch.float64, device=DEV)
    for n, J, status in ((64, 65, 6), (1 << 31, 4, 6), (0, 4, 2), (64, 0, 3)):
        with pytest.raises(B.Int8tError) as e:
            B.int8t_dsgc_clip_static(g, n, rd, J, B.ROUND_STOCHASTIC, 0, clip, d)
        assert e.value.status == status
    with pytest.raises(B.Int8tError) as e:
        B.int8t_dsgc_clip_static(None, 64, rd, 4, B.ROUND_STOCHASTIC, 0, clip, d)
    assert e.value.status == 1
