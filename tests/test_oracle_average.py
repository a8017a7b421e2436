"""Pins for the oracle's gated average (Sec. 3.1, eq. "average") with per-coordinate loads."""
import numpy as np
import torch

import workloads


def _bf16_bits(a):
    return workloads.bf16_bits(torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16))


def test_full_coverage_is_the_plain_mean(orc):
    # m = m^uni (C = 1): the gated average is data parallelism's mean over the n workers
    rng = np.random.default_rng(0)
    K, R, D = 5, 7, 9
    g = [rng.standard_normal((R, D)) for _ in range(K)]
    out, cov = orc.gated_average(g, np.ones((K, R), dtype=np.uint8))
    assert (cov == K).all()
    np.testing.assert_allclose(out, sum(g) / K, rtol=1e-15, atol=1e-15)


def test_brute_force_on_tiny_mask_sets(orc):
    rng = np.random.default_rng(1)
    for K, R, D in [(1, 3, 2), (2, 4, 3), (3, 5, 1), (8, 16, 4)]:
        for trial in range(20):
            mask = (rng.random((K, R)) < 0.5).astype(np.uint8)
            g = [rng.standard_normal((R, D)) for _ in range(K)]
            out, cov = orc.gated_average(g, mask)
            for r in range(R):
                who = [k for k in range(K) if mask[k, r]]
                assert cov[r] == len(who)
                for e in range(D):
                    want = sum(g[k][r, e] for k in who) / len(who) if who else 0.0
                    assert abs(out[r, e] - want) <= 1e-15 * max(1.0, abs(want))


def test_single_worker_is_identity_on_its_mask_and_zero_elsewhere(orc):
    rng = np.random.default_rng(2)
    g = [rng.standard_normal((6, 4))]
    mask = np.array([[1, 0, 1, 1, 0, 1]], dtype=np.uint8)
    out, cov = orc.gated_average(g, mask)
    assert (out[mask[0] == 1] == g[0][mask[0] == 1]).all()
    assert (out[mask[0] == 0] == 0.0).all() and (cov == mask[0]).all()


def test_constant_gradients_average_to_the_constant(orc):
    K, R, D = 6, 40, 3
    mask = orc.make_masks(K, R, 10, 3, False)
    g = [np.full((R, D), 0.375) for _ in range(K)]
    out, cov = orc.gated_average(g, mask)
    assert (out[cov > 0] == 0.375).all() and (out[cov == 0] == 0.0).all()
    assert (cov == 0).any() and (cov > 1).any()


def test_off_mask_entries_are_never_read(orc):
    # the mask selects: NaN in rows a worker does not cover must not reach the result
    rng = np.random.default_rng(3)
    K, R, D = 4, 30, 5
    mask = orc.make_masks(K, R, 12, 8, False)
    g = [rng.standard_normal((R, D)).astype(np.float32) for _ in range(K)]
    clean, cov = orc.gated_average(g, mask)
    poisoned = [x.copy() for x in g]
    for k in range(K):
        poisoned[k][mask[k] == 0] = np.nan
    out, cov2 = orc.gated_average(poisoned, mask)
    assert np.isfinite(out).all() and (out == clean).all() and (cov == cov2).all()


def test_linearity_and_dtype_widening(orc):
    rng = np.random.default_rng(4)
    K, R, D = 3, 11, 8
    mask = orc.make_masks(K, R, 6, 2, True)
    a = [rng.standard_normal((R, D)) for _ in range(K)]
    b = [rng.standard_normal((R, D)) for _ in range(K)]
    oa, _ = orc.gated_average(a, mask)
    ob, _ = orc.gated_average(b, mask)
    oc, _ = orc.gated_average([2.0 * x - 3.0 * y for x, y in zip(a, b)], mask)
    np.testing.assert_allclose(oc, 2.0 * oa - 3.0 * ob, rtol=1e-13, atol=1e-13)
    # bf16 bit patterns widen exactly: same result as feeding the bf16 values as fp64
    bits = [_bf16_bits(x) for x in a]
    vals = [torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy() for x in a]
    o1, _ = orc.gated_average(bits, mask)
    o2, _ = orc.gated_average(vals, mask)
    assert (o1 == o2).all()
    o3, _ = orc.gated_average([v.astype(np.float32) for v in vals], mask)
    assert (o3 == o2).all()


def test_sdp_step_at_coverage_one_equals_ddp(orc):
    # whole step, Sec. 3.1: with the all-ones mask both regimes give per-worker dense gradients
    # and their gated average is the DDP mean
    rng = np.random.default_rng(5)
    K, T, d, F = 3, 6, 4, 5
    W1, W3, W2T = (rng.standard_normal((F, d)) * 0.5 for _ in range(3))
    ones = np.ones((K, F), dtype=np.uint8)
    grads = {"fm": [], "bm": []}
    dense = []
    for k in range(K):
        X, dY = rng.standard_normal((T, d)), rng.standard_normal((T, d))
        f = orc.mlp_fwd(X, W1, W3, W2T)
        dense.append(orc.mlp_bwd(X, dY, W1, W3, W2T, f["G"], f["U"], f["A"])["dW1"])
        for mode in grads:
            grads[mode].append(orc.worker_step(mode, ones[k], X, dY, W1, W3, W2T)["dW1"])
    for mode in grads:
        out, cov = orc.gated_average(grads[mode], ones)
        np.testing.assert_allclose(out, sum(dense) / K, rtol=1e-15, atol=1e-15)


def test_squared_norm_of_the_average(orc):
    """The quantity global gradient clipping measures (App. "Hyperparameters for LLM Architecture")."""
    rng = np.random.default_rng(21)
    K, R, D = 6, 40, 11
    mask = (rng.random((K, R)) < 0.5).astype(np.uint8)
    mask[:, :3] = 0  # rows nobody covers
    g = [rng.standard_normal((R, D)) for _ in range(K)]
    out, cov = orc.gated_average(g, mask)
    got = orc.gated_average_sqnorm(g, mask)
    # a library norm of the average that is pinned on its own above
    assert abs(got - np.linalg.norm(out) ** 2) <= 1e-12 * got
    # uncovered rows count for nothing, even when their buffers hold garbage
    g2 = [a.copy() for a in g]
    for a in g2:
        a[:3] = np.nan
    assert orc.gated_average_sqnorm(g2, mask) == got
    # one worker that holds everything: the plain sum of squares; scaling the gradients by a scales it by a^2
    assert abs(orc.gated_average_sqnorm(g[:1], np.ones((1, R), np.uint8)) - (g[0] ** 2).sum()) <= 1e-12 * (g[0] ** 2).sum()
    assert abs(orc.gated_average_sqnorm([3.0 * a for a in g], mask) - 9.0 * got) <= 1e-12 * got
    # constant gradients v on every covered row: v^2 D (number of covered rows), whatever the loads
    const = [np.full((R, D), -1.5) for _ in range(K)]
    assert abs(orc.gated_average_sqnorm(const, mask) - 2.25 * D * int((mask.sum(axis=0) > 0).sum())) < 1e-9
    # hand-computed: two workers, rows of load 2, 1, 0
    m = np.array([[1, 1, 0], [1, 0, 0]], dtype=np.uint8)
    a = [np.array([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]]), np.array([[3.0, 0.0], [7.0, 7.0], [7.0, 7.0]])]
    # averages: row 0 -> (2, 1), row 1 -> (3, 4), row 2 -> 0
    assert orc.gated_average_sqnorm(a, m) == 4.0 + 1.0 + 9.0 + 16.0
    # bf16 bit patterns widen exactly
    gb = [np.asarray(_bf16_bits(x)) for x in g]
    gw = [torch.from_numpy(np.asarray(x, dtype=np.float32)).to(torch.bfloat16).double().numpy() for x in g]
    assert orc.gated_average_sqnorm(gb, mask) == orc.gated_average_sqnorm(gw, mask)
