"""Pins for the oracle's head-masked attention block (Sec. 4.1: heads masked on W_Q, W_K, W_V, W_O).

The dense block is checked against a library routine (torch's scaled_dot_product_attention in fp64, with
autograd for every gradient), against central finite differences, and against what the definitions fix:
causality, a softmax that averages, and a sequence of one token.  Head masking is checked against what
Sec. 3.1 fixes: C = 1 is the dense block, a forward-masked worker is the physically smaller block made of
its heads alone, and the gradient of every head it does not hold is exactly zero.
"""
import numpy as np
import pytest
import torch


def _setup(seed, Bt, S, d, H, hd, wscale=0.3):
    rng = np.random.default_rng(seed)
    T, E = Bt * S, H * hd
    return dict(
        X=rng.standard_normal((T, d)), dY=rng.standard_normal((T, d)),
        Wq=rng.standard_normal((E, d)) * wscale, Wk=rng.standard_normal((E, d)) * wscale,
        Wv=rng.standard_normal((E, d)) * wscale, WoT=rng.standard_normal((E, d)) * wscale,
    )


def _dense(orc, Bt, S, hd, s):
    f = orc.attn_fwd(Bt, S, hd, s["X"], s["Wq"], s["Wk"], s["Wv"], s["WoT"])
    b = orc.attn_bwd(Bt, S, hd, s["X"], s["dY"], s["Wq"], s["Wk"], s["Wv"], s["WoT"], f["Q"], f["K"], f["V"], f["O"])
    return f, b


def _torch_block(Bt, S, H, hd, s):
    t = {k: torch.tensor(v, dtype=torch.float64, requires_grad=(k != "dY")) for k, v in s.items()}
    T = Bt * S

    def heads(z):
        return z.view(Bt, S, H, hd).transpose(1, 2)

    q, k, v = (heads(t["X"] @ t[w].T) for w in ("Wq", "Wk", "Wv"))
    o = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
    o = o.transpose(1, 2).reshape(T, H * hd)
    y = o @ t["WoT"]
    (y * t["dY"]).sum().backward()
    return y.detach().numpy(), o.detach().numpy(), {k: t[k].grad.numpy() for k in ("X", "Wq", "Wk", "Wv", "WoT")}


@pytest.mark.parametrize("Bt,S,d,H,hd", [(1, 7, 5, 2, 3), (3, 20, 24, 4, 8), (2, 33, 16, 3, 16)])
def test_dense_block_matches_library_attention_and_autograd(orc, Bt, S, d, H, hd):
    s = _setup(3, Bt, S, d, H, hd)
    f, b = _dense(orc, Bt, S, hd, s)
    y, o, g = _torch_block(Bt, S, H, hd, s)
    np.testing.assert_allclose(f["O"], o, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(f["Y"], y, rtol=1e-11, atol=1e-12)
    for name, gname in (("X", "dX"), ("Wq", "dWq"), ("Wk", "dWk"), ("Wv", "dWv"), ("WoT", "dWoT")):
        np.testing.assert_allclose(b[gname], g[name], rtol=1e-10, atol=1e-11, err_msg=gname)


def test_dense_gradients_match_central_differences(orc):
    Bt, S, d, H, hd = 2, 4, 3, 2, 2
    s = _setup(4, Bt, S, d, H, hd, wscale=0.7)
    _, b = _dense(orc, Bt, S, hd, s)

    def loss(a):
        return float((orc.attn_fwd(Bt, S, hd, a["X"], a["Wq"], a["Wk"], a["Wv"], a["WoT"])["Y"] * a["dY"]).sum())

    h = 1e-5
    for name, gname in (("X", "dX"), ("Wq", "dWq"), ("Wk", "dWk"), ("Wv", "dWv"), ("WoT", "dWoT")):
        fd = np.zeros_like(s[name])
        for i in np.ndindex(*s[name].shape):
            plus, minus = s[name].copy(), s[name].copy()
            plus[i] += h
            minus[i] -= h
            fd[i] = (loss(dict(s, **{name: plus})) - loss(dict(s, **{name: minus}))) / (2 * h)
        np.testing.assert_allclose(b[gname], fd, rtol=2e-6, atol=2e-8, err_msg=gname)


def test_causal_and_per_sequence(orc):
    """A token's output depends on the tokens before it in its own sequence, and on nothing else."""
    Bt, S, d, H, hd = 2, 9, 6, 2, 4
    s = _setup(5, Bt, S, d, H, hd)
    y0 = orc.attn_fwd(Bt, S, hd, s["X"], s["Wq"], s["Wk"], s["Wv"], s["WoT"])["Y"]
    X = s["X"].copy()
    X[5] += 1.0  # sequence 0, position 5
    y1 = orc.attn_fwd(Bt, S, hd, X, s["Wq"], s["Wk"], s["Wv"], s["WoT"])["Y"]
    changed = np.abs(y1 - y0).max(axis=1) > 0
    assert not changed[:5].any() and changed[5:S].all() and not changed[S:].any()


def test_softmax_averages_and_single_token(orc):
    Bt, S, d, H, hd = 1, 6, 4, 2, 3
    s = _setup(6, Bt, S, d, H, hd)
    # identical tokens: every value row is the same, so any convex combination returns it
    X = np.tile(s["X"][:1], (S, 1))
    f = orc.attn_fwd(Bt, S, hd, X, s["Wq"], s["Wk"], s["Wv"], s["WoT"])
    np.testing.assert_allclose(f["O"], f["V"], rtol=1e-13, atol=1e-14)
    # zero queries: uniform weights over the causal prefix -> running mean of V
    f = orc.attn_fwd(Bt, S, hd, s["X"], 0 * s["Wq"], s["Wk"], s["Wv"], s["WoT"])
    want = np.cumsum(f["V"], axis=0) / np.arange(1, S + 1)[:, None]
    np.testing.assert_allclose(f["O"], want, rtol=1e-12, atol=1e-13)
    # sequences of one token: O = V
    f = orc.attn_fwd(S, 1, hd, s["X"], s["Wq"], s["Wk"], s["Wv"], s["WoT"])
    np.testing.assert_allclose(f["O"], f["V"], rtol=0, atol=0)
    # the logits are scaled by 1 / sqrt(hd): two tokens, one head, hand-computed weights
    Xs = np.array([[1.0, 0.0], [0.0, 1.0]])
    eye = np.eye(2)
    Wq = np.array([[0.0, 3.0], [0.0, 0.0]])  # q_1 = (3, 0), q_0 = 0
    Wk = np.array([[2.0, 1.0], [0.0, 0.0]])  # k_0 = (2, 0), k_1 = (1, 0)
    f = orc.attn_fwd(1, 2, 2, Xs, Wq, Wk, eye, eye)
    z = np.array([6.0, 3.0]) / np.sqrt(2.0)
    w = np.exp(z) / np.exp(z).sum()
    np.testing.assert_allclose(f["O"][1], w[0] * Xs[0] + w[1] * Xs[1], rtol=1e-14)
    np.testing.assert_allclose(f["O"][0], Xs[0], rtol=0)


def test_full_head_mask_is_the_dense_block(orc):
    Bt, S, d, H, hd = 2, 10, 8, 3, 4
    s = _setup(7, Bt, S, d, H, hd)
    f, b = _dense(orc, Bt, S, hd, s)
    r = orc.attn_worker_step(Bt, S, hd, np.ones(H, np.uint8), s["X"], s["dY"], s["Wq"], s["Wk"], s["Wv"], s["WoT"])
    for name in ("Q", "K", "V", "O", "Y"):
        assert (r[name] == f[name]).all()
    for name in ("dX", "dWq", "dWk", "dWv", "dWoT"):
        assert (r[name] == b[name]).all()


@pytest.mark.parametrize("held", [[0], [1, 3], [0, 2, 3]])
def test_forward_masked_worker_is_the_block_of_its_heads(orc, held):
    """The worker's subnetwork is the dense block built from the held heads' rows alone; the rows of the
    other heads receive an exactly zero gradient."""
    Bt, S, d, H, hd = 2, 12, 10, 4, 4
    s = _setup(8, Bt, S, d, H, hd)
    mask = np.zeros(H, np.uint8)
    mask[held] = 1
    r = orc.attn_worker_step(Bt, S, hd, mask, s["X"], s["dY"], s["Wq"], s["Wk"], s["Wv"], s["WoT"])
    assert r["nonzero_off_mask"] == 0
    rows = np.concatenate([np.arange(h * hd, (h + 1) * hd) for h in held])
    small = dict(s, **{w: s[w][rows] for w in ("Wq", "Wk", "Wv", "WoT")})
    f, b = _dense(orc, Bt, S, hd, small)
    np.testing.assert_allclose(r["Y"], f["Y"], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(r["O"][:, rows], f["O"], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(r["dX"], b["dX"], rtol=1e-12, atol=1e-13)
    off = np.setdiff1d(np.arange(H * hd), rows)
    for name in ("dWq", "dWk", "dWv", "dWoT"):
        np.testing.assert_allclose(r[name][rows], b[name], rtol=1e-12, atol=1e-13, err_msg=name)
        assert (r[name][off] == 0).all()
    # and it differs from the dense block
    dense, _ = _dense(orc, Bt, S, hd, s)
    assert np.abs(dense["Y"] - r["Y"]).max() > 1e-3


@pytest.mark.parametrize("held", [[2], [0, 3]])
def test_backward_masked_worker_sees_the_dense_block(orc, held):
    """Backward masking (m_fwd = all ones, m_bwd = m): outputs and dX are those of the dense block, the weight
    gradient is the dense one on the held heads' rows and zero elsewhere; with every head held both regimes
    coincide with the dense block."""
    Bt, S, d, H, hd = 2, 11, 9, 4, 4
    s = _setup(9, Bt, S, d, H, hd)
    mask = np.zeros(H, np.uint8)
    mask[held] = 1
    f, b = _dense(orc, Bt, S, hd, s)
    r = orc.attn_worker_step(Bt, S, hd, mask, s["X"], s["dY"], s["Wq"], s["Wk"], s["Wv"], s["WoT"], mode="bm")
    for name in ("Q", "K", "V", "O", "Y"):
        assert (r[name] == f[name]).all()
    assert (r["dX"] == b["dX"]).all()
    rows = np.concatenate([np.arange(h * hd, (h + 1) * hd) for h in held])
    off = np.setdiff1d(np.arange(H * hd), rows)
    for name in ("dWq", "dWk", "dWv", "dWoT"):
        assert (r[name][rows] == b[name][rows]).all()
        assert (r[name][off] == 0).all() and np.abs(b[name][off]).max() > 0
    assert r["nonzero_off_mask"] == 0  # nothing is counted in this regime
    full = orc.attn_worker_step(Bt, S, hd, np.ones(H, np.uint8), s["X"], s["dY"], s["Wq"], s["Wk"], s["Wv"], s["WoT"], mode="bm")
    for name in ("Y", "dX", "dWq", "dWk", "dWv", "dWoT"):
        assert (full[name] == (f[name] if name == "Y" else b[name])).all()
    # the two regimes differ in Y and dX as soon as a head is not held; for a given upstream gradient dY the
    # heads do not interact, so the held heads' weight gradients are the same under both
    fm = orc.attn_worker_step(Bt, S, hd, mask, s["X"], s["dY"], s["Wq"], s["Wk"], s["Wv"], s["WoT"], mode="fm")
    assert np.abs(fm["Y"] - r["Y"]).max() > 1e-3 and np.abs(fm["dX"] - r["dX"]).max() > 1e-3
    for name in ("dWq", "dWk", "dWv", "dWoT"):
        np.testing.assert_allclose(fm[name][rows], r[name][rows], rtol=1e-13, atol=1e-15)
