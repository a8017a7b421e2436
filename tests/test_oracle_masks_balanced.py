"""Pins for the oracle's balanced mask construction (App. A, Algorithm "Structured Mask Construction").

The paper prints no worked example, so the pins are what the text fixes: the exact row budget, the
target load t = ceil(K p / F), the objective (max_j |c_j - K p / F| small), the behaviour of the
weights max(t - c_j, eps) in the cases where they force the outcome, and the stopping rule of the
repair phase re-derived here by brute force.
"""
import numpy as np
import pytest

CASES = [(4, 1024, 512), (4, 4096, 2048), (8, 688, 516), (3, 100, 41), (5, 64, 64), (6, 97, 13), (2, 50, 1)]


def loads(m):
    return m.astype(np.int64).sum(axis=0)


@pytest.mark.parametrize("K,F,p", CASES)
def test_row_budget_binary_deterministic(orc, K, F, p):
    a = orc.make_masks_balanced(K, F, p, 11)
    assert set(np.unique(a)) <= {0, 1}
    assert (a.astype(np.int64).sum(axis=1) == p).all()  # App. A: sum_j M_ij = p for every worker
    assert np.array_equal(a, orc.make_masks_balanced(K, F, p, 11))
    if 0 < p < F:
        assert not np.array_equal(a, orc.make_masks_balanced(K, F, p, 12))


@pytest.mark.parametrize("K,F,p", [(4, 64, 16), (2, 50, 25), (8, 1024, 128), (3, 99, 33)])
def test_partition_when_budget_equals_components(orc, K, F, p):
    # K p = F, so t = 1: a worker's weights are 1 on the columns nobody holds and eps = 1e-6 on the rest; the
    # chance that any of the K p draws lands on a held column is below 1e-3, and the repair phase would undo it
    for seed in range(20):
        m = orc.make_masks_balanced(K, F, p, seed)
        assert (loads(m) == 1).all()


@pytest.mark.parametrize("K,F,p", [(4, 1024, 512), (8, 512, 128), (6, 96, 32), (4, 4096, 2048)])
def test_exact_balance_when_target_is_reachable(orc, K, F, p):
    # K p = t F: the objective's minimum (every c_j = t) is reachable; the construction reaches it
    t = K * p // F
    assert K * p == t * F
    for seed in (1, 2, 3):
        assert (loads(orc.make_masks_balanced(K, F, p, seed)) == t).all()


@pytest.mark.parametrize("K,F,p", CASES[:4] + [(8, 5504, 4128)])
def test_imbalance_not_worse_than_uniform(orc, K, F, p):
    # the objective of App. A: max_j |c_j - K p / F|; compare with the uniform sampler on the same sizes
    mean = K * p / F
    for seed in (5, 6):
        bal = np.abs(loads(orc.make_masks_balanced(K, F, p, seed)) - mean).max()
        uni = np.abs(loads(orc.make_masks(K, F, p, seed, False)) - mean).max()
        assert bal <= uni


@pytest.mark.parametrize("K,F,p", CASES)
def test_repair_stopping_rule(orc, K, F, p):
    # phase 2 may stop on a column only when no worker qualifies: re-derive "qualifies" here by brute force
    m = orc.make_masks_balanced(K, F, p, 3)
    c = loads(m)
    t = -(-K * p // F)
    for j in np.nonzero(c < t)[0]:
        for i in range(K):
            if m[i, j]:
                continue
            held = np.nonzero(m[i])[0]
            assert not (c[held] > t).any(), (i, j)


def test_single_worker_is_uniform(orc):
    # K = 1: all loads are 0, all weights equal, so the p columns are a uniform random p-subset
    F, p, N = 12, 4, 6000
    counts = np.zeros(F)
    for seed in range(N):
        counts += orc.make_masks_balanced(1, F, p, seed)[0]
    expect = N * p / F
    chi2 = ((counts - expect) ** 2 / (expect * (1 - p / F))).sum()
    assert chi2 < 40.0  # 11 degrees of freedom: 40 is far beyond the 0.999 quantile (31.3)


def test_weights_follow_deficit(orc):
    # two workers, K p / F = 1.5 so t = 2: for worker 1 the u = 2 columns worker 0 lacks weigh 2 (deficit 2),
    # the h = 6 it holds weigh 1.  Successive draws with renormalisation: P(next pick is a lacking column)
    # = 2u / (2u + h).  The probability that both lacking columns are among worker 1's six picks follows by
    # recursion over (u, h, draws left); no load can exceed t = 2 with two workers, so phase 2 changes nothing
    # and "the two masks together cover all 8 columns" happens with exactly that probability.
    from functools import lru_cache

    @lru_cache(None)
    def p_all(u, h, left):
        if u == 0:
            return 1.0
        if left == 0:
            return 0.0
        tot = 2 * u + h
        out = 2 * u / tot * p_all(u - 1, h, left - 1)
        if h:
            out += h / tot * p_all(u, h - 1, left - 1)
        return out

    K, F, p, N = 2, 8, 6, 6000
    expect = p_all(2, 6, 6)
    hits = sum(int((m[0] | m[1]).all()) for m in (orc.make_masks_balanced(K, F, p, seed) for seed in range(N)))
    sigma = (expect * (1 - expect) / N) ** 0.5
    assert abs(hits / N - expect) < 4.5 * sigma, (hits / N, expect)
    # the same experiment with equal weights would give C(6,4)/C(8,6) = 15/28 = 0.536: the weights matter
    assert abs(expect - 15 / 28) > 10 * sigma


def test_degenerate_budgets(orc):
    assert orc.make_masks_balanced(3, 10, 0, 1).sum() == 0
    assert (orc.make_masks_balanced(3, 10, 10, 1) == 1).all()
    with pytest.raises(ValueError):
        orc.make_masks_balanced(3, 10, 11, 1)
