"""GPU parity at the full benchmark sizes (configs 2-5), on sampled outputs.

The oracle cannot compute 1e12-1e13 fp64 flop in a test, but every output element it is asked for
it computes exactly as at small size:
  - a token row of Y, dX, G, U depends only on that row of X, dY: the oracle runs the whole
    worker step on a sample of rows (first / last rows of the first and last tiles included);
  - the weight-gradient rows of neuron j depend only on neuron j's weights (and all tokens): the
    oracle runs the dense block restricted to a sample of the worker's active neurons over all T
    tokens (first / last active neurons and the ragged last tile included).
The launch configuration is the one bench.py times (same entry points, same layouts).
"""
import numpy as np
import pytest
import torch

import workloads
from helpers import assert_close

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2


@pytest.fixture(scope="module")
def sdp():
    import paper_2507_09029_amd as m

    assert torch.cuda.is_available()
    m.lib()
    return m


def _sample(n, count, rng, always):
    pick = set(int(x) for x in always if 0 <= x < n)
    pick.update(int(x) for x in rng.choice(n, size=min(count, n), replace=False))
    return np.array(sorted(pick))


def _fullsize_worker(sdp, orc, w, k, Wd, W64, idx, want_mask, dw_layout):
    rng = np.random.default_rng(1000 + k)
    X, dY = workloads.mlp_batch(w, k)
    Xd, dYd = X.cuda(), dY.cuda()
    Y, G, U = sdp.masked_mlp_fwd(w.mode, Xd, *Wd, idx[k])
    dX, dW1, dW3, dW2T = sdp.masked_mlp_bwd(w.mode, Xd, dYd, *Wd, idx[k], G, U, dw_layout=dw_layout)
    torch.cuda.synchronize()
    S = np.flatnonzero(want_mask[k])

    # token-row sample: tile edges (tiles of 128 / 256 rows), the very last rows, random rows
    rows = _sample(w.T, 256, rng, [0, 1, 127, 128, 255, 256, w.T - 257, w.T - 256, w.T - 129, w.T - 128, w.T - 2, w.T - 1])
    assert len(rows) >= 256
    X64, dY64 = workloads.to_f64(X), workloads.to_f64(dY)
    ref = orc.worker_step(w.mode, want_mask[k], X64[rows], dY64[rows], *W64)
    cols = S if w.mode == "fm" else np.arange(w.F)
    trows = torch.from_numpy(rows).cuda()
    assert_close(workloads.to_f64(Y[trows]), ref["Y"], TOL_BF16, f"{w.name} Y[{k}]")
    assert_close(workloads.to_f64(dX[trows]), ref["dX"], TOL_BF16, f"{w.name} dX[{k}]")
    assert_close(workloads.to_f64(G[trows]), ref["G"][:, cols], TOL_BF16, f"{w.name} G[{k}]")
    assert_close(workloads.to_f64(U[trows]), ref["U"][:, cols], TOL_BF16, f"{w.name} U[{k}]")

    # neuron sample among the worker's active neurons, by rank: tile edges and the ragged tail
    p = len(S)
    ranks = _sample(p, 64, rng, [0, 1, 31, 32, 127, 128, 255, 256, p - 130, p - 129, p - 33, p - 32, p - 2, p - 1])
    assert len(ranks) >= 64
    neurons = S[ranks]
    f = orc.mlp_fwd(X64, W64[0][neurons], W64[1][neurons], W64[2][neurons])
    b = orc.mlp_bwd(X64, dY64, W64[0][neurons], W64[1][neurons], W64[2][neurons], f["G"], f["U"], f["A"])
    sel = torch.from_numpy(neurons if dw_layout == "scatter" else ranks).cuda()
    for name, got in (("dW1", dW1), ("dW3", dW3), ("dW2T", dW2T)):
        assert_close(workloads.to_f64(got[sel]), b[name], TOL_BF16, f"{w.name} {name}[{k}]")
    del Y, G, U, dX, dW1, dW3, dW2T, Xd, dYd
    torch.cuda.empty_cache()


@pytest.mark.parametrize("w", [workloads.CONFIG2, workloads.CONFIG3, workloads.CONFIG4], ids=["config2", "config3", "config4"])
def test_fullsize_mlp_sampled(sdp, orc, w):
    """Every worker of the configuration (each has its own index list and its own batch): at least 256 token rows
    and at least 64 of its neurons; the two gradient layouts alternate from worker to worker."""
    W = workloads.mlp_weights(w)
    Wd = [t.cuda() for t in W]
    W64 = [workloads.to_f64(t) for t in W]
    mask, idx, pos, cov = sdp.make_masks(w.K, w.F, w.p, w.mask_seed, True)
    want_mask = orc.make_masks(w.K, w.F, w.p, w.mask_seed, True)
    assert (mask.cpu().numpy() == want_mask).all()
    widx, wpos, wcount, wcov = orc.index_masks(want_mask, idx_ld=w.p)
    assert (idx.cpu().numpy() == widx).all() and (cov.cpu().numpy() == wcov).all()
    for k in range(w.K):
        layout = ("compact", "scatter")[k % 2]
        print(f"  {w.name}: worker {k}, layout {layout}", flush=True)
        _fullsize_worker(sdp, orc, w, k, Wd, W64, idx, want_mask, layout)


def test_fullsize_config5_average_sampled(sdp, orc):
    c = workloads.CONFIG5
    print(f"  {c.name}: K={c.K} R={c.R} D={c.D} p={c.p}", flush=True)
    want_mask = orc.make_masks(c.K, c.R, c.p, c.mask_seed, False)
    mask = sdp.sample_masks_host(c.K, c.R, c.p, c.mask_seed, False)
    assert (mask.numpy() == want_mask).all()
    dmask = mask.cuda()
    # off-mask rows hold NaN: a correct average never reads them
    grads = workloads.grad_buffers(c.K, c.R, c.D, c.sigma, "bf16", device="cuda", poison_mask=dmask)
    out, cov = sdp.coverage_grad_avg(grads, dmask)
    torch.cuda.synchronize()
    _, _, wcount, wcov = orc.index_masks(want_mask, idx_ld=1)
    assert (wcount == c.p).all()
    assert (cov.cpu().numpy() == wcov).all()                       # every count, bit exact
    assert bool(torch.isfinite(out).all())                         # at full size: nothing off-mask was read
    uncovered = np.flatnonzero(wcov == 0)
    assert len(uncovered) > 0                                      # the workload does exercise c = 0
    assert bool((out[torch.from_numpy(uncovered).cuda()] == 0).all())
    rng = np.random.default_rng(5)
    rows = _sample(c.R, 1500, rng, list(uncovered[:50]) + [0, 1, 2, 3, 4, c.R - 4, c.R - 3, c.R - 2, c.R - 1])
    trows = torch.from_numpy(rows).cuda()
    sub = [workloads.bf16_bits(g[trows]) for g in grads]
    want, wc = orc.gated_average(sub, want_mask[:, rows])
    assert (wc == wcov[rows]).all()
    assert_close(out[trows].cpu().numpy(), want, 1e-5, "config5 average (sampled rows)")


def test_fullsize_config5_squared_norm(sdp, orc):
    """The norm pass at config 5 in bench.py's launch configuration: it must equal the norm of the stored average
    (whose elements the test above samples against the oracle) to fp64 summation error, repeat bit for bit, and
    match the oracle's own norm on a slice of rows that the oracle finishes in seconds."""
    c = workloads.CONFIG5
    mask_host = sdp.sample_masks_host(c.K, c.R, c.p, c.mask_seed, False)
    mask = mask_host.cuda()
    grads = workloads.grad_buffers(c.K, c.R, c.D, c.sigma, "bf16", device="cuda")
    print(f"fullsize sqnorm K={c.K} R={c.R} D={c.D}", flush=True)
    a = sdp.coverage_grad_sqnorm(grads, mask)
    b = sdp.coverage_grad_sqnorm(grads, mask)
    out, cov = sdp.coverage_grad_avg(grads, mask)
    torch.cuda.synchronize()
    got = float(a.cpu()[0])
    assert got == float(b.cpu()[0]) and got > 0.0
    stored = 0.0
    for r0 in range(0, c.R, 1 << 16):  # in pieces: an fp64 copy of the whole average would not be a small tensor
        stored += float((out[r0:r0 + (1 << 16)].double() ** 2).sum().cpu())
    assert abs(got - stored) <= 1e-11 * stored
    rows = slice(1000, 3000)
    part = sdp.coverage_grad_sqnorm([g[rows] for g in grads], mask[:, rows].contiguous())
    torch.cuda.synchronize()
    want = orc.gated_average_sqnorm([workloads.bf16_bits(g[rows]) for g in grads], mask_host[:, rows].numpy())
    assert abs(float(part.cpu()[0]) - want) <= 1e-5 * want


def test_fullsize_config5_adamw_sampled(sdp, orc):
    """The fused average + AdamW pass at the 1B-parameter size, sampled rows against the oracle."""
    c = workloads.CONFIG5
    hp = dict(lr=4e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    print(f"  {c.name} + AdamW: K={c.K} R={c.R} D={c.D} p={c.p}", flush=True)
    want_mask = orc.make_masks(c.K, c.R, c.p, c.mask_seed, False)
    dmask = torch.from_numpy(want_mask).cuda()
    grads = workloads.grad_buffers(c.K, c.R, c.D, c.sigma, "bf16", device="cuda", poison_mask=dmask)
    gen = torch.Generator(device="cuda").manual_seed(99)
    theta = torch.randn((c.R, c.D), generator=gen, device="cuda") * 0.02
    m = torch.randn((c.R, c.D), generator=gen, device="cuda") * 1e-4
    v = (torch.randn((c.R, c.D), generator=gen, device="cuda") * 1e-4) ** 2
    _, _, _, wcov = orc.index_masks(want_mask, idx_ld=1)
    uncovered = np.flatnonzero(wcov == 0)
    rng = np.random.default_rng(6)
    rows = _sample(c.R, 1200, rng, list(uncovered[:50]) + [0, 1, 2, 3, c.R - 3, c.R - 2, c.R - 1])
    trows = torch.from_numpy(rows).cuda()
    before = [t[trows].cpu().numpy() for t in (theta, m, v)]
    cov = sdp.coverage_avg_adamw(grads, dmask, theta, m, v, step=12, **hp)
    torch.cuda.synchronize()
    assert (cov.cpu().numpy() == wcov).all()
    assert bool(torch.isfinite(theta).all()) and bool(torch.isfinite(m).all()) and bool(torch.isfinite(v).all())
    sub = [workloads.bf16_bits(g[trows]) for g in grads]
    wth, wm, wv, wc = orc.avg_adamw(sub, want_mask[:, rows], *before, step=12, **hp)
    got = [t[trows].cpu().numpy() for t in (theta, m, v)]
    off = wc == 0
    for b, g_ in zip(before, got):
        assert (g_[off] == b[off]).all()                           # uncovered rows: state untouched, bit for bit
    assert_close(got[1], wm, 1e-5, "config5 AdamW m (sampled rows)")
    assert_close(got[2], wv, 1e-5, "config5 AdamW v (sampled rows)")
    assert_close(got[0], wth, 1e-5, "config5 AdamW theta (sampled rows)")
    assert_close(got[0].astype(np.float64) - before[0], wth - before[0], 1e-4, "config5 AdamW update (sampled rows)")


def test_attention_500M_one_sequence_and_sampled_gradient_rows(sdp, orc):
    """Head-masked attention block at the size bench.py times (4 sequences of 2048 tokens, 12 of 24 heads).

    Sequences do not interact: the oracle runs the dense block made of the worker's held heads on the last
    sequence alone (all of Y, O and dX of that sequence are compared).  A weight-gradient row sums over all
    tokens: the oracle's per-sequence gradients are summed over the four sequences for the held heads' rows of
    one head (first and last row blocks included).
    """
    from helpers import assert_close_rows

    w = workloads.ATTN_500M
    Wqkv, WoT = workloads.attn_weights(w)
    mask, idx, pos, cov = sdp.make_masks(w.K, w.H, w.ph, w.mask_seed, True)
    want_mask = orc.make_masks(w.K, w.H, w.ph, w.mask_seed, True)
    assert (mask.cpu().numpy() == want_mask).all()
    k = w.K - 1
    heads = np.flatnonzero(want_mask[k])
    rows = np.concatenate([np.arange(h * w.hd, (h + 1) * w.hd) for h in heads])
    E = rows.size
    X, dY = workloads.attn_batch(w, k)
    print(f"  {w.name} worker {k}: GPU forward + backward", flush=True)
    Y, QKV, O, LSE = sdp.masked_attn_fwd("fm", w.Bt, w.S, w.hd, X.cuda(), Wqkv.cuda(), WoT.cuda(), idx[k])
    dX, gWqkv, gWoT = sdp.masked_attn_bwd("fm", w.Bt, w.S, w.hd, X.cuda(), dY.cuda(), Wqkv.cuda(), WoT.cuda(), idx[k], QKV, O, LSE)
    torch.cuda.synchronize()
    Wc = [workloads.to_f64(Wqkv[i])[rows] for i in range(3)] + [workloads.to_f64(WoT)[rows]]
    X64, dY64 = workloads.to_f64(X), workloads.to_f64(dY)
    gq = np.zeros((E, w.d)); gk = np.zeros((E, w.d)); gv = np.zeros((E, w.d)); go = np.zeros((E, w.d))
    for b in range(w.Bt):
        print(f"  oracle: sequence {b}", flush=True)
        sl = slice(b * w.S, (b + 1) * w.S)
        f = orc.attn_fwd(1, w.S, w.hd, X64[sl], *Wc)
        r = orc.attn_bwd(1, w.S, w.hd, X64[sl], dY64[sl], *Wc, f["Q"], f["K"], f["V"], f["O"])
        gq += r["dWq"]; gk += r["dWk"]; gv += r["dWv"]; go += r["dWoT"]
        if b == w.Bt - 1:
            assert_close_rows(workloads.to_f64(Y[sl]), f["Y"], TOL_BF16, "Y")
            assert_close_rows(workloads.to_f64(O[sl]), f["O"], TOL_BF16, "O")
            assert_close_rows(workloads.to_f64(dX[sl]), r["dX"], TOL_BF16, "dX")
    g = workloads.to_f64(gWqkv)
    for i, (name, want) in enumerate((("dWq", gq), ("dWk", gk), ("dWv", gv))):
        assert_close(g[i], want, TOL_BF16, name, elem_tol=3e-2)
    assert_close(workloads.to_f64(gWoT), go, TOL_BF16, "dWoT", elem_tol=3e-2)
