"""GPU parity of AdaptiveSpeculation (spec_adaptive_speculation, through the C ABI) against the CPU
oracle's sequential loop: exact integer equality over random pools, budgets around every regime
(under budget, partial level, everything at one), batch masks, and sizes that span several
1024-request chunks of the index-ordered assignment."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sv():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2503_10325_amd import binding
    binding.lib()
    return binding


def run(sv, gamma, budget, mask=None):
    t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    g = t(gamma)
    out = torch.full_like(g, -7)
    total = torch.zeros(1, dtype=torch.int64, device="cuda")
    sv.spec_adaptive_speculation(g, budget, out, in_batch=t(mask), total_out=total)
    torch.cuda.synchronize()
    return out.cpu().numpy(), int(total.item())


@pytest.mark.parametrize("R", [1, 7, 64, 1000, 1024, 1025, 5000])
@pytest.mark.parametrize("masked", [False, True])
def test_adaptive_matches_sequential_loop(sv, R, masked):
    rng = np.random.default_rng(R + 17 * masked)
    gamma = rng.integers(1, 11, size=R).astype(np.int32)        # the serving workload draws k in 2..10
    mask = (rng.random(R) < 0.7).astype(np.int32) if masked else None
    tot = int(gamma.sum() if mask is None else gamma[mask != 0].sum())
    for budget in sorted({0, 1, tot // 4, tot // 2, tot - 3, tot - 1, tot, tot + 9}):
        got, got_total = run(sv, gamma, budget, mask)
        want, want_total = oracle.adaptive_speculation(gamma, budget, mask)
        assert np.array_equal(got, want), (R, budget)
        assert got_total == want_total


def test_adaptive_ties_and_odd_values(sv):
    # ties go to the lowest index; values below 1 are left alone
    got, total = run(sv, [8, 8, 8, 8], 29)
    assert got.tolist() == [7, 7, 7, 8] and total == 29
    got, total = run(sv, [5, 0, 9, -2, 9], 12)
    want, want_total = oracle.adaptive_speculation([5, 0, 9, -2, 9], 12)
    assert got.tolist() == want.tolist() and total == want_total
