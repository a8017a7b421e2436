"""Pins for the oracle's random numbers, mask sampler, index form and coverage counts.

None of these re-call the oracle to check itself: they use published generator
outputs, invariants the paper states for the mask matrix (Sec. 3.1, App. A:
exact row budget p, column loads c_j), brute force and a uniformity statistic.
"""
import itertools
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
GOLDEN_GAMMA = 0x9E3779B97F4A7C15
M64 = 2**64 - 1


def test_mix64_matches_published_splitmix64_sequence(orc):
    want = [int(l, 16) for l in open(os.path.join(GOLDEN, "splitmix64_seed0.txt")) if not l.startswith("#")]
    got = [orc.mix64(((i + 1) * GOLDEN_GAMMA) & M64) for i in range(len(want))]
    assert got == want


def test_rand64_is_counter_based_and_streams_differ(orc):
    a = [orc.rand64(7, 0, c) for c in range(64)]
    assert a == [orc.rand64(7, 0, c) for c in range(64)]
    assert len(set(a)) == 64
    assert orc.rand64(7, 1, 0) != orc.rand64(7, 0, 0)
    assert orc.rand64(8, 0, 0) != orc.rand64(7, 0, 0)
    # keyed construction written out with python integers
    key = orc.mix64((7 + GOLDEN_GAMMA * (3 + 1)) & M64)
    assert orc.rand64(7, 3, 5) == orc.mix64((key + GOLDEN_GAMMA * (5 + 1)) & M64)


def test_bounded_draw_rejects_the_biased_tail(orc):
    # n = 3 * 2^62: 2^64 mod n = 2^62, so a quarter of raw draws are rejected and the counter skips them
    n = 3 * 2**62
    ctr, rejected = 0, 0
    for _ in range(400):
        before = ctr
        v, ctr = orc.rand_below(11, 0, ctr, n)
        raws = [orc.rand64(11, 0, c) for c in range(before, ctr)]
        assert all(r < 2**62 for r in raws[:-1]) and raws[-1] >= 2**62
        assert v == raws[-1] % n and 0 <= v < n
        rejected += len(raws) - 1
    assert 60 < rejected < 220  # expectation 400/3
    # small n: plain residue of the first raw draw, values spread over all residues
    vals = []
    ctr = 0
    for _ in range(3000):
        before = ctr
        v, ctr = orc.rand_below(5, 2, ctr, 6)
        assert ctr == before + 1 and v == orc.rand64(5, 2, before) % 6
        vals.append(v)
    counts = np.bincount(vals, minlength=6)
    chi2 = ((counts - 500.0) ** 2 / 500.0).sum()
    assert chi2 < 25.0  # 5 dof, p ~ 1e-4


@pytest.mark.parametrize("K,F,p", [(4, 1024, 512), (4, 4096, 2048), (8, 5504, 4128), (3, 7, 3), (2, 10, 5), (8, 64, 8)])
def test_mask_invariants_with_cover(orc, K, F, p):
    m = orc.make_masks(K, F, p, 1234, True)
    assert m.dtype == np.uint8 and set(np.unique(m)) <= {0, 1}
    assert (m.sum(axis=1) == p).all()  # exact row budget (App. A)
    load = m.astype(np.int64).sum(axis=0)
    assert load.min() >= 1 and load.max() <= K
    assert load.sum() == K * p
    assert (m == orc.make_masks(K, F, p, 1234, True)).all()  # same seed, same bits
    assert (m != orc.make_masks(K, F, p, 1235, True)).any()
    if p < F and K > 1:
        assert any((m[0] != m[k]).any() for k in range(1, K))  # workers use different streams


def test_mask_without_cover_keeps_budget_and_is_a_prefix_of_the_covered_one(orc):
    K, F, p = 4, 1024, 512
    raw = orc.make_masks(K, F, p, 99, False)
    fixed = orc.make_masks(K, F, p, 99, True)
    assert (raw.sum(axis=1) == p).all()
    uncovered = np.flatnonzero(raw.sum(axis=0) == 0)
    assert len(uncovered) > 20  # (1/2)^4 * 1024 = 64 expected
    # the repair moves exactly one assignment per uncovered neuron and touches nothing else
    assert (raw != fixed).sum() == 2 * len(uncovered)
    assert (fixed[:, uncovered].sum(axis=0) == 1).all()
    removed = np.argwhere((raw == 1) & (fixed == 0))
    raw_load = raw.astype(np.int64).sum(axis=0)
    assert (raw_load[removed[:, 1]] >= 2).all()  # only donors with load >= 2 give up a neuron


def test_mask_error_paths(orc):
    with pytest.raises(ValueError):
        orc.make_masks(2, 10, 4, 1, True)  # K p < F: coverage impossible
    with pytest.raises(ValueError):
        orc.make_masks(2, 10, 11, 1, False)  # p > F
    m = orc.make_masks(2, 10, 5, 1, True)  # K p == F: must be a partition
    assert (m.sum(axis=0) == 1).all()
    assert (orc.make_masks(3, 9, 9, 1, True) == 1).all()  # C = 1: all-ones mask (DDP)
    assert (orc.make_masks(3, 9, 0, 1, False) == 0).all()


def test_sampler_is_uniform_over_neurons(orc):
    # each neuron is picked by a worker with probability p/F: chi-square over many seeds
    K, F, p, seeds = 4, 32, 8, 600
    counts = np.zeros(F)
    pair = np.zeros((F, F))
    for s in range(seeds):
        m = orc.make_masks(K, F, p, 1000 + s, False).astype(np.float64)
        counts += m.sum(axis=0)
        pair += m.T @ m
    n = seeds * K
    expect = n * p / F
    var = n * (p / F) * (1 - p / F)
    chi2 = ((counts - expect) ** 2 / var).sum()
    assert chi2 < 75.0, chi2  # ~31 dof; p(chi2 > 75) ~ 2e-5
    # pairs: P(i and j both picked) = p(p-1) / (F(F-1)) for a uniform p-subset
    off = pair[~np.eye(F, dtype=bool)]
    expect2 = n * p * (p - 1) / (F * (F - 1))
    assert abs(off.mean() - expect2) < 1e-9 * n + 1e-6  # exact by counting: sum is n p (p-1)
    assert np.abs(off - expect2).max() < 6 * np.sqrt(expect2)


def test_first_draw_of_partial_shuffle_follows_the_stream(orc):
    # worker k's first chosen neuron is perm[0] after one swap: index rand_below(stream k, F)
    K, F = 5, 97
    m = orc.make_masks(K, F, 1, 4242, False)
    for k in range(K):
        v, _ = orc.rand_below(4242, k, 0, F)
        assert np.flatnonzero(m[k]).tolist() == [v]


def _brute_index(mask):
    K, F = mask.shape
    idx = [[j for j in range(F) if mask[k, j]] for k in range(K)]
    cov = [sum(int(mask[k, j]) for k in range(K)) for j in range(F)]
    return idx, cov


def test_index_and_coverage_exhaustive_tiny(orc):
    # every row-budgeted mask matrix for K <= 3, F <= 5
    for K, F in [(1, 3), (2, 4), (3, 4), (2, 5)]:
        for p in range(0, F + 1):
            rows = [np.array([1 if j in c else 0 for j in range(F)], dtype=np.uint8) for c in itertools.combinations(range(F), p)]
            for combo in itertools.product(range(len(rows)), repeat=K):
                mask = np.stack([rows[i] for i in combo])
                idx, pos, count, cov = orc.index_masks(mask, idx_ld=max(p, 1))
                bidx, bcov = _brute_index(mask)
                assert cov.tolist() == bcov
                assert count.tolist() == [p] * K
                for k in range(K):
                    assert idx[k, :p].tolist() == bidx[k]
                    assert (idx[k, p:] == -1).all()
                    want_pos = [-1] * F
                    for i, j in enumerate(bidx[k]):
                        want_pos[j] = i
                    assert pos[k].tolist() == want_pos


def test_index_random_and_ragged(orc):
    rng = np.random.default_rng(5)
    for K, F in [(8, 64), (5, 333), (1, 1), (3, 4097)]:
        mask = (rng.random((K, F)) < 0.4).astype(np.uint8)
        mask[0] = 0  # an empty worker
        if K > 1:
            mask[1] = 1  # a full worker
        idx, pos, count, cov = orc.index_masks(mask, idx_ld=F)
        assert cov.tolist() == mask.astype(np.int64).sum(axis=0).tolist()
        for k in range(K):
            want = np.flatnonzero(mask[k])
            assert count[k] == len(want)
            assert (idx[k, : len(want)] == want).all() and (idx[k, len(want):] == -1).all()
            assert (np.diff(idx[k, : len(want)]) > 0).all()
            assert (pos[k, want] == np.arange(len(want))).all()
            assert (pos[k, mask[k] == 0] == -1).all()


def test_rho2_closed_form_for_constant_load(orc):
    # constant column load c: rho^2 = |J| (1/c - 1/n) (distance to uniform masking, Thm. 3.1)
    K, F = 4, 12
    mask = np.zeros((K, F), dtype=np.uint8)
    for j in range(F):
        mask[j % K, j] = 1
        mask[(j + 1) % K, j] = 1
    assert abs(orc.rho2(mask) - F * (1 / 2 - 1 / K)) < 1e-12
    assert orc.rho2(np.ones((K, F), dtype=np.uint8)) == 0.0  # C = 1 is DDP


def test_rho2_by_hand_and_against_a_library_norm(orc):
    # two workers, three columns of load 2, 1, 0: the entries of (1/n) 1 - m / c are
    #   column 0: 0, 0;  column 1: -1/2, 1/2;  column 2 (nobody holds it): 1/2, 1/2  ->  rho^2 = 0 + 1/2 + 1/2
    assert orc.rho2(np.array([[1, 1, 0], [1, 0, 0]], dtype=np.uint8)) == 1.0
    # uneven loads: the matrix written out and handed to numpy's Frobenius norm
    rng = np.random.default_rng(12)
    K, F = 7, 301
    mask = (rng.random((K, F)) < 0.4).astype(np.uint8)
    mask[:, :5] = 0
    c = mask.sum(axis=0)
    A = np.full((K, F), 1.0 / K) - np.divide(mask, c, out=np.zeros((K, F)), where=c > 0)
    assert abs(orc.rho2(mask) - np.linalg.norm(A, "fro") ** 2) < 1e-10
    # transposing the roles of the two terms' signs or dropping the uncovered columns would show here
    assert abs(orc.rho2(mask) - np.linalg.norm(A[:, 5:], "fro") ** 2 - 5 / K) < 1e-10
