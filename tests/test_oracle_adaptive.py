"""Pins of the oracle's AdaptiveSpeculation (Algorithm 2) against what the loop must produce:
worked examples, the water-filling closed form computed independently by sorting, invariants
(budget met or everything at 1, nothing increases, reduced requests end within one token of each
other, ties to the lowest index, requests outside the batch untouched)."""
import numpy as np
import pytest

import oracle


def waterfill(gamma, budget, mask=None):
    """Independent closed form: lower the tallest columns to a common level; the last partial level
    goes to the lowest indices first."""
    g = np.array(gamma, dtype=np.int64)
    idx = np.arange(len(g)) if mask is None else np.flatnonzero(np.asarray(mask) != 0)
    sub = g[idx].copy()
    need = int(sub.sum()) - int(budget)
    if need <= 0:
        return g
    need = min(need, int(np.maximum(sub - 1, 0).sum()))
    level = int(sub.max())
    while need > 0:                                     # peel whole levels off the columns above `level - 1`
        tall = np.flatnonzero(sub >= level)
        if level <= 1:
            break
        if len(tall) <= need:
            sub[tall] = level - 1
            need -= len(tall)
            level -= 1
        else:
            sub[tall[:need]] = level - 1                # lowest indices first
            need = 0
    g[idx] = sub
    return g


def test_worked_examples():
    out, total = oracle.adaptive_speculation([5, 3, 8, 8], 20)
    # 24 -> 20: decrements hit index 2, 3 (8,8 -> 7,7), then 2, 3 again (6,6)
    assert out.tolist() == [5, 3, 6, 6] and total == 20
    out, total = oracle.adaptive_speculation([5, 3, 8, 8], 21)
    assert out.tolist() == [5, 3, 6, 7] and total == 21    # tie at 7: the lowest index gives first
    out, total = oracle.adaptive_speculation([4, 4, 4], 100)
    assert out.tolist() == [4, 4, 4] and total == 12       # under budget: untouched
    out, total = oracle.adaptive_speculation([3, 2, 1], 1)
    assert out.tolist() == [1, 1, 1] and total == 3        # everyone keeps one token
    out, total = oracle.adaptive_speculation([9, 9, 9], 20, in_batch=[1, 0, 1])
    assert out.tolist() == [9, 9, 9] and total == 18
    out, total = oracle.adaptive_speculation([9, 9, 9], 10, in_batch=[1, 0, 1])
    assert out.tolist() == [5, 9, 5] and total == 10


@pytest.mark.parametrize("seed", range(6))
def test_matches_waterfilling_closed_form(seed):
    rng = np.random.default_rng(seed)
    R = int(rng.integers(1, 200))
    gamma = rng.integers(1, 12, size=R).astype(np.int32)
    mask = None if seed % 2 == 0 else (rng.random(R) < 0.7).astype(np.int32)
    tot = int(gamma.sum() if mask is None else gamma[mask != 0].sum())
    for budget in (0, tot // 3, tot // 2, tot - 1, tot, tot + 5):
        out, total = oracle.adaptive_speculation(gamma, budget, mask)
        want = waterfill(gamma, budget, mask)
        assert np.array_equal(out, want)
        sel = np.ones(R, bool) if mask is None else mask != 0
        assert total == int(out[sel].sum())
        assert np.all(out <= gamma) and np.all(out[sel] >= np.minimum(gamma[sel], 1))
        assert total <= budget or np.all(out[sel] <= 1)
        changed = sel & (out < gamma)
        if changed.any():
            assert out[changed].max() - out[changed].min() <= 1
            assert out[sel].max() <= out[changed].min() + 1     # nothing left more than one above a reduced one
