"""Pins for the oracle's SwiGLU MLP, forward masking and backward masking.

The dense forward is checked against a library contraction, the gradients
against central finite differences of L = <dY, Y>, and the two masking regimes
against what Sec. 3.1 / 3.2 fix: C = 1 is plain data parallelism, a forward-masked
worker is the physically smaller dense network, its off-mask gradient is exactly
zero, and a backward-masked worker sees the dense loss and the dense gradient
restricted to its mask.
"""
import numpy as np
import pytest


def _rand(rng, *shape, scale=1.0):
    return rng.standard_normal(shape) * scale


def _silu(z):
    return z / (1.0 + np.exp(-z))


def _setup(seed, T, d, F, wscale=0.5):
    rng = np.random.default_rng(seed)
    return dict(
        X=_rand(rng, T, d), dY=_rand(rng, T, d),
        W1=_rand(rng, F, d, scale=wscale), W3=_rand(rng, F, d, scale=wscale), W2T=_rand(rng, F, d, scale=wscale),
    )


@pytest.mark.parametrize("T,d,F", [(5, 7, 11), (33, 16, 40), (64, 96, 130)])
def test_dense_forward_matches_einsum(orc, T, d, F):
    s = _setup(1, T, d, F)
    r = orc.mlp_fwd(s["X"], s["W1"], s["W3"], s["W2T"])
    G = np.einsum("te,je->tj", s["X"], s["W1"])
    U = np.einsum("te,je->tj", s["X"], s["W3"])
    A = _silu(G) * U
    Y = np.einsum("tj,je->te", A, s["W2T"])
    for name, want in (("G", G), ("U", U), ("A", A), ("Y", Y)):
        np.testing.assert_allclose(r[name], want, rtol=1e-12, atol=1e-12)
    # W1 and W3 are not interchangeable: the gate goes through silu, the other branch is linear
    r2 = orc.mlp_fwd(s["X"], s["W3"], s["W1"], s["W2T"])
    assert np.abs(r2["Y"] - Y).max() > 1e-3


def _loss(orc, s, **over):
    a = dict(s, **over)
    return float((orc.mlp_fwd(a["X"], a["W1"], a["W3"], a["W2T"])["Y"] * a["dY"]).sum())


def test_dense_gradients_match_central_differences(orc):
    T, d, F = 4, 5, 6
    s = _setup(2, T, d, F)
    f = orc.mlp_fwd(s["X"], s["W1"], s["W3"], s["W2T"])
    b = orc.mlp_bwd(s["X"], s["dY"], s["W1"], s["W3"], s["W2T"], f["G"], f["U"], f["A"])
    h = 1e-5
    for name, gname in (("X", "dX"), ("W1", "dW1"), ("W3", "dW3"), ("W2T", "dW2T")):
        base = s[name]
        fd = np.zeros_like(base)
        for i in np.ndindex(*base.shape):
            plus = base.copy(); plus[i] += h
            minus = base.copy(); minus[i] -= h
            fd[i] = (_loss(orc, s, **{name: plus}) - _loss(orc, s, **{name: minus})) / (2 * h)
        scale = np.abs(fd).max()
        assert np.abs(b[gname] - fd).max() < 2e-8 * max(scale, 1.0), gname
    # the intermediate gradients: dL/dG and dL/dU by differencing A -> Y directly
    dA = s["dY"] @ s["W2T"].T
    np.testing.assert_allclose(b["dU"], dA * _silu(f["G"]), rtol=1e-12, atol=1e-13)
    eps = 1e-6
    dsilu = (_silu(f["G"] + eps) - _silu(f["G"] - eps)) / (2 * eps)
    np.testing.assert_allclose(b["dG"], dA * f["U"] * dsilu, rtol=1e-7, atol=1e-8)


def test_coverage_one_reduces_both_regimes_to_the_dense_mlp(orc):
    T, d, F = 9, 8, 12
    s = _setup(3, T, d, F)
    ones = np.ones(F, dtype=np.uint8)
    f = orc.mlp_fwd(s["X"], s["W1"], s["W3"], s["W2T"])
    b = orc.mlp_bwd(s["X"], s["dY"], s["W1"], s["W3"], s["W2T"], f["G"], f["U"], f["A"])
    for mode in ("fm", "bm"):
        w = orc.worker_step(mode, ones, s["X"], s["dY"], s["W1"], s["W3"], s["W2T"])
        for name in ("G", "U", "Y"):
            assert (w[name] == f[name]).all(), (mode, name)
        for name in ("dX", "dW1", "dW3", "dW2T"):
            assert (w[name] == b[name]).all(), (mode, name)


def test_forward_masking_is_the_smaller_dense_network(orc):
    # Sec. 3.2: removing neuron j removes row j of W1/W3 and column j of W2; the gated full-size
    # network and the physically compact one give the same outputs and gradients
    T, d, F = 17, 10, 24
    s = _setup(4, T, d, F)
    mask = orc.make_masks(3, F, 9, 77, True)[1]
    S = np.flatnonzero(mask)
    w = orc.worker_step("fm", mask, s["X"], s["dY"], s["W1"], s["W3"], s["W2T"])
    assert w["nonzero_off_mask"] == 0  # (m_fwd)_ij = 0  =>  (g_i)_j = 0, exactly
    off = np.flatnonzero(mask == 0)
    for name in ("dW1", "dW3", "dW2T"):
        assert (w[name][off] == 0.0).all()
    # compact route: slice first, then run the small dense MLP
    fc = orc.mlp_fwd(s["X"], s["W1"][S], s["W3"][S], s["W2T"][S])
    bc = orc.mlp_bwd(s["X"], s["dY"], s["W1"][S], s["W3"][S], s["W2T"][S], fc["G"], fc["U"], fc["A"])
    np.testing.assert_allclose(w["Y"], fc["Y"], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(w["dX"], bc["dX"], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(w["G"][:, S], fc["G"], rtol=0, atol=0)
    np.testing.assert_allclose(w["U"][:, S], fc["U"], rtol=0, atol=0)
    assert (w["G"][:, off] == 0).all() and (w["U"][:, off] == 0).all()
    for name in ("dW1", "dW3", "dW2T"):
        np.testing.assert_allclose(w[name][S], bc[name], rtol=1e-13, atol=1e-13)
    # gating only the first layer is already enough: (m W^l, W^{l+1}) == (m W^l, m W^{l+1})
    W1g = s["W1"] * mask[:, None]
    W3g = s["W3"] * mask[:, None]
    half = orc.mlp_fwd(s["X"], W1g, W3g, s["W2T"])
    np.testing.assert_allclose(half["Y"], w["Y"], rtol=1e-13, atol=1e-13)
    # and the masked network differs from the dense one
    dense = orc.mlp_fwd(s["X"], s["W1"], s["W3"], s["W2T"])
    assert np.abs(dense["Y"] - w["Y"]).max() > 1e-2


def test_forward_masking_gradient_is_the_gradient_of_the_masked_loss(orc):
    # finite differences of the loss evaluated at the gated parameters (Sec. 3.1), w.r.t. full parameters
    T, d, F = 3, 4, 6
    s = _setup(5, T, d, F)
    mask = np.array([1, 0, 1, 1, 0, 0], dtype=np.uint8)
    w = orc.worker_step("fm", mask, s["X"], s["dY"], s["W1"], s["W3"], s["W2T"])

    def masked_loss(a):
        y = orc.mlp_fwd(a["X"], a["W1"] * mask[:, None], a["W3"] * mask[:, None], a["W2T"] * mask[:, None])["Y"]
        return float((y * a["dY"]).sum())

    h = 1e-5
    for name, gname in (("X", "dX"), ("W1", "dW1"), ("W3", "dW3"), ("W2T", "dW2T")):
        fd = np.zeros_like(s[name])
        for i in np.ndindex(*s[name].shape):
            plus = s[name].copy(); plus[i] += h
            minus = s[name].copy(); minus[i] -= h
            fd[i] = (masked_loss(dict(s, **{name: plus})) - masked_loss(dict(s, **{name: minus}))) / (2 * h)
        assert np.abs(w[gname] - fd).max() < 2e-8 * max(np.abs(fd).max(), 1.0), gname


def test_backward_masking_is_dense_forward_with_restricted_weight_gradient(orc):
    T, d, F = 13, 6, 20
    s = _setup(6, T, d, F)
    mask = orc.make_masks(4, F, 10, 5, True)[2]
    f = orc.mlp_fwd(s["X"], s["W1"], s["W3"], s["W2T"])
    b = orc.mlp_bwd(s["X"], s["dY"], s["W1"], s["W3"], s["W2T"], f["G"], f["U"], f["A"])
    w = orc.worker_step("bm", mask, s["X"], s["dY"], s["W1"], s["W3"], s["W2T"])
    # m_fwd = m^uni: activations, output and dX are those of the full network for every worker
    for name in ("G", "U", "Y"):
        assert (w[name] == f[name]).all()
    assert (w["dX"] == b["dX"]).all()
    # m_bwd = m: the weight gradient is the dense one on the mask and absent elsewhere
    for name in ("dW1", "dW3", "dW2T"):
        assert (w[name] == b[name] * mask[:, None]).all()
        assert np.abs(b[name][mask == 0]).min() > 0  # the dense gradient there is not zero
    # with dY fixed, a neuron's own weight gradient does not depend on the other neurons, so on the mask
    # both regimes agree; they differ in what flows on: the output and the input gradient
    wf = orc.worker_step("fm", mask, s["X"], s["dY"], s["W1"], s["W3"], s["W2T"])
    np.testing.assert_allclose(wf["dW1"], w["dW1"], rtol=1e-13, atol=1e-13)
    assert np.abs(wf["Y"] - w["Y"]).max() > 1e-3 and np.abs(wf["dX"] - w["dX"]).max() > 1e-3


def test_per_row_and_per_neuron_slices_are_exact(orc):
    # the sliced protocol used at full size: a token row of Y/dX depends only on that row of X/dY,
    # a neuron's weight-gradient rows only on that neuron's weights (backward masking / dense case)
    T, d, F = 12, 6, 10
    s = _setup(7, T, d, F)
    f = orc.mlp_fwd(s["X"], s["W1"], s["W3"], s["W2T"])
    b = orc.mlp_bwd(s["X"], s["dY"], s["W1"], s["W3"], s["W2T"], f["G"], f["U"], f["A"])
    rows = [0, 5, 11]
    fr = orc.mlp_fwd(s["X"][rows], s["W1"], s["W3"], s["W2T"])
    br = orc.mlp_bwd(s["X"][rows], s["dY"][rows], s["W1"], s["W3"], s["W2T"], fr["G"], fr["U"], fr["A"])
    assert (fr["Y"] == f["Y"][rows]).all() and (br["dX"] == b["dX"][rows]).all()
    nz = [2, 3, 9]
    fn = orc.mlp_fwd(s["X"], s["W1"][nz], s["W3"][nz], s["W2T"][nz])
    bn = orc.mlp_bwd(s["X"], s["dY"], s["W1"][nz], s["W3"][nz], s["W2T"][nz], fn["G"], fn["U"], fn["A"])
    for name in ("dW1", "dW3", "dW2T"):
        assert (bn[name] == b[name][nz]).all()
