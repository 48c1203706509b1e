"""GPU parity of the error-bound estimator (Sections 4.1-4.3) against the oracle.

Bar: R is a ratio of two integers, Lbar a mean of exact maxima, so both agree to the last bits of
an fp64 sum taken in another order (relative 1e-12); Mavg is an fp64 sum of up to millions of fp32
magnitudes in another order (relative 1e-10); the bound itself is those three through Eq. 8 in
fp64, rounded once to fp32: one unit in the last place (relative 1.2e-7).
"""
import numpy as np
import pytest
import torch

from paper_2011_09017_amd.workloads import activation

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2011_09017_amd import binding
    binding.lib()
    return binding


def check(gpu, orc, ctx, act, loss, mom, **kw):
    rc, eb, (R, Lbar, Mavg) = ctx.estimate_eb(torch.from_numpy(act).cuda(), torch.from_numpy(loss).cuda(),
                                               torch.from_numpy(mom).cuda(), **kw)
    orc_rc, oeb, (oR, oL, oM) = orc.estimate_eb(act, loss, mom, **kw)
    assert rc == orc_rc
    assert R == oR
    if np.isfinite(oL):
        assert Lbar == pytest.approx(oL, rel=1e-12)
    else:
        assert not np.isfinite(Lbar)
    if np.isfinite(oM):
        assert Mavg == pytest.approx(oM, rel=1e-10)
    assert eb == pytest.approx(float(oeb), rel=1.2e-7)
    return eb


CASES = [
    # activation shape, loss shape, momentum size
    ((8, 16, 28, 28), (8, 16, 28, 28), 16 * 16 * 9),
    ((3, 5, 7, 11), (3, 5, 7, 11), 77),                 # per-sample size not a multiple of 4, ragged tails
    ((1, 1, 1, 1), (1, 1), 1),
    ((64, 64, 56, 56), (64, 64, 56, 56), 64 * 64 * 9),  # several slices per array
    ((4, 3, 5, 5), (300, 8), 4099),                     # many short samples
]


@pytest.mark.parametrize("ashape,lshape,nmom", CASES)
def test_estimate_matches_oracle(gpu, orc, ashape, lshape, nmom):
    rng = np.random.default_rng(hash((ashape, lshape, nmom)) % (1 << 32))
    act = np.maximum(rng.standard_normal(ashape), 0).astype(np.float32)
    loss = (rng.standard_normal(lshape) * 1e-3).astype(np.float32)
    mom = (rng.standard_normal(nmom) * 1e-2).astype(np.float32)
    ctx = gpu.Context(max_numel=1 << 16)
    check(gpu, orc, ctx, act, loss, mom)
    check(gpu, orc, ctx, act, loss, mom, sigma_frac=0.05, a=0.5, eb_min=1e-3, eb_max=2e-3)   # clamped; scratch re-armed


def test_degenerate_inputs_and_reuse(gpu, orc):
    ctx = gpu.Context(max_numel=1 << 16)
    one = np.ones((2, 1, 2, 2), np.float32)
    loss = np.ones((2, 4), np.float32)
    mom = np.ones(4, np.float32)
    nan_mid = loss.copy()
    nan_mid[1, 1] = np.nan
    for a_, l_, m_ in ((0 * one, loss, mom), (one, 0 * loss, mom), (one, nan_mid, mom), (one, loss, mom * np.inf),
                       (one, loss, mom)):                                   # the last one: an ordinary call after them
        check(gpu, orc, ctx, a_, l_, m_, eb_min=1e-4)
    assert gpu.cmp_estimate_eb(ctx._h, 0, 4, 0, 1, 4, 0, 4, None, 0)[0] == gpu.CMP_E_ARG


def test_on_a_config5_activation(gpu, orc):
    """The second tensor of the ResNet-18 stream as activation and (scaled) as loss."""
    act = activation((256, 64, 56, 56), 5, 0.5, 201109017, device="cuda")
    loss = (act * 1e-4).roll(1, 0).contiguous()
    mom = act[0, :8].contiguous() * 1e-2
    ctx = gpu.Context(max_numel=1 << 16)
    rc, eb, stats = ctx.estimate_eb(act, loss, mom)
    orc_rc, oeb, ostats = orc.estimate_eb(act.cpu().numpy(), loss.cpu().numpy(), mom.cpu().numpy())
    assert rc == orc_rc == 0
    assert stats[0] == ostats[0]
    assert stats[1] == pytest.approx(ostats[1], rel=1e-12) and stats[2] == pytest.approx(ostats[2], rel=1e-10)
    assert eb == pytest.approx(float(oeb), rel=1.2e-7)
