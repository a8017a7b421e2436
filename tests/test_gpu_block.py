"""GPU parity of the block-level calls (Sec. 3.2: masked block m B(x) + x; backward-masked variant) against the
fp64 oracle: every element of Y, dX and the seven weight gradients of one block, the skipped cases bit for bit,
and a K-worker step over a stack of blocks whose block-granular gradient buffers go through the coverage average
(one mask byte per block)."""
import numpy as np
import pytest
import torch

import rounding_model as rm
from helpers import assert_close, assert_close_rows, assert_close_with_model

pytestmark = pytest.mark.gpu

NAMES = ("Wq", "Wk", "Wv", "WoT", "W1", "W3", "W2T")


@pytest.fixture(scope="module")
def sdp():
    import paper_2507_09029_amd as m

    assert torch.cuda.is_available()
    m.lib()
    return m


def _setup(seed, Bt, S, d, H, hd, F, dtype):
    g = torch.Generator().manual_seed(seed)
    T, E = Bt * S, H * hd
    dt = torch.float32 if dtype == "f32" else torch.bfloat16

    def draw(shape, std):
        return (torch.randn(shape, generator=g) * std).to(dt)

    t = dict(X=draw((T, d), 1.0), dY=draw((T, d), 1.0), Wqkv=draw((3, E, d), 0.05), WoT=draw((E, d), 0.05),
             W1=draw((F, d), 0.05), W3=draw((F, d), 0.05), W2T=draw((F, d), 0.05))
    return t


def _f64(t):
    return t.to(torch.float64).numpy()


def _oracle_weights(t):
    return [_f64(t["Wqkv"][i]) for i in range(3)] + [_f64(t[n]) for n in ("WoT", "W1", "W3", "W2T")]


def _check_grads(got, ref, tol, dw_elem):
    dWqkv, dWoT, dW1, dW3, dW2T = [_f64(x.cpu()) for x in got]
    for i, n in enumerate(("dWq", "dWk", "dWv")):
        assert_close(dWqkv[i], ref[n], tol, n, elem_tol=dw_elem)
    assert_close(dWoT, ref["dWoT"], tol, "dWoT", elem_tol=dw_elem)
    for n, g in (("dW1", dW1), ("dW3", dW3), ("dW2T", dW2T)):
        assert_close(g, ref[n], tol, n, elem_tol=dw_elem)


CASES = [
    ("f32", 2, 40, 48, 3, 16, 96),      # plain kernels everywhere, ragged sizes
    ("bf16", 2, 256, 256, 4, 64, 512),  # MFMA contractions and MFMA attention core
    ("bf16", 1, 200, 128, 2, 64, 264),  # ragged sequence and hidden width
    ("bf16", 2, 96, 64, 2, 32, 128),    # head width the MFMA core does not take: plain core
    ("bf16", 2, 200, 200, 4, 50, 520),  # the paper's head width (padded to 64 inside), ragged everything
]


@pytest.mark.parametrize("dtype,Bt,S,d,H,hd,F", CASES)
@pytest.mark.parametrize("mode,m,rule", [("fm", 1, "through"), ("bm", 1, "through"), ("bm", 0, "through"), ("bm", 0, "skip"), ("fm", 0, "through")])
def test_block_matches_oracle(sdp, orc, dtype, Bt, S, d, H, hd, F, mode, m, rule):
    print(f"block {dtype} Bt={Bt} S={S} d={d} H={H} hd={hd} F={F} mode={mode} m={m} dx_rule={rule}", flush=True)
    tol = 1e-5 if dtype == "f32" else 2e-2
    # weight gradients behind the attention core and two stacked halves: same elementwise allowance as the attention tests
    dw_elem = None if dtype == "f32" else 3e-2
    t = _setup(100 + S + F, Bt, S, d, H, hd, F, dtype)
    c = {k: v.cuda() for k, v in t.items()}
    W = (c["Wqkv"], c["WoT"], c["W1"], c["W3"], c["W2T"])
    ref = orc.block_step(mode, m, Bt, S, hd, _f64(t["X"]), _f64(t["dY"]), *_oracle_weights(t), dx_rule=rule)
    Y, saved = sdp.block_fwd(mode, m, Bt, S, hd, c["X"], *W)
    dX, grads = sdp.block_bwd(mode, m, Bt, S, hd, c["X"], c["dY"], *W, saved, dx_rule=rule)
    torch.cuda.synchronize()
    if ref["computed"] == "skipped":
        assert saved is None and grads is None
        assert torch.equal(Y, c["X"]) and torch.equal(dX, c["dY"])  # bit for bit
        return
    if dtype == "f32":
        assert_close_rows(_f64(Y.cpu()), ref["Y"], tol, "Y")
        if ref["computed"] == "forward only" and rule == "skip":
            assert grads is None and torch.equal(dX, c["dY"])
            return
        assert_close_rows(_f64(dX.cpu()), ref["dX"], tol, "dX")
        if m:
            _check_grads(grads, ref, tol, None)
        else:
            assert grads is None
        return
    # bf16: two halves are chained, so the second one's inputs already carry the first one's rounding error.  Every
    # tensor is held to the oracle at 2e-2 normwise, and its error figures may not exceed what the bf16 rounding
    # points alone produce (the rounding model) by more than the slack of assert_close_with_model; the fixed bound on
    # the elementwise maximum is 2e-2 for Y, 3e-2 for dX (two chained halves) and 4e-2 for the weight gradients.
    mod = rm.block_model(mode, m, Bt, S, hd, _f64(t["X"]), _f64(t["dY"]), *_oracle_weights(t), dx_rule=rule)
    assert_close_with_model(_f64(Y.cpu()), mod["Y"], ref["Y"], tol, "Y", rows=True)
    a = orc.attn_fwd(Bt, S, hd, _f64(t["X"]), *_oracle_weights(t)[:4])
    assert_close_with_model(_f64(saved[0].cpu()), mod["Hm"], _f64(t["X"]) + a["Y"], tol, "Hm", rows=True)
    if ref["computed"] == "forward only" and rule == "skip":
        assert grads is None and torch.equal(dX, c["dY"])
        return
    assert_close_with_model(_f64(dX.cpu()), mod["dX"], ref["dX"], tol, "dX", rows=True, elem_allow=3e-2)
    if not m:
        assert grads is None
        return
    dWqkv, dWoT, dW1, dW3, dW2T = [_f64(x.cpu()) for x in grads]
    for n, g in (("dWq", dWqkv[0]), ("dWk", dWqkv[1]), ("dWv", dWqkv[2]), ("dWoT", dWoT), ("dW1", dW1), ("dW3", dW3), ("dW2T", dW2T)):
        assert_close_with_model(g, mod[n], ref[n], tol, n, elem_allow=4e-2)


def test_masked_block_leaves_gradient_buffers_alone(sdp):
    """Backward masking, m = 0, gradient carried through the block: the weight-gradient buffers are not written."""
    Bt, S, d, H, hd, F = 1, 128, 128, 2, 64, 256
    t = _setup(7, Bt, S, d, H, hd, F, "bf16")
    c = {k: v.cuda() for k, v in t.items()}
    W = (c["Wqkv"], c["WoT"], c["W1"], c["W3"], c["W2T"])
    Y, saved = sdp.block_fwd("bm", 0, Bt, S, hd, c["X"], *W)
    E = H * hd
    poison = [torch.full(s, float("nan"), dtype=torch.bfloat16, device="cuda") for s in ((3, E, d), (E, d), (F, d), (F, d), (F, d))]
    out = (torch.empty_like(c["X"]), *poison)
    L = sdp.lib()
    ws = torch.empty(sdp.block_bwd_workspace_bytes(torch.bfloat16, Bt, S, d, H, hd, F), dtype=torch.uint8, device="cuda")
    Hm, QKV, O, LSE, G, U = saved
    st = L.sdp_block_bwd(1, 0, 0, 1, Bt, S, d, H, hd, F, c["X"].data_ptr(), c["dY"].data_ptr(), *[w.data_ptr() for w in W],
                         Hm.data_ptr(), QKV.data_ptr(), O.data_ptr(), LSE.data_ptr(), G.data_ptr(), U.data_ptr(),
                         out[0].data_ptr(), *[p.data_ptr() for p in poison], ws.data_ptr(), ws.numel(), None)
    torch.cuda.synchronize()
    assert st == 0
    assert bool(torch.isfinite(out[0]).all())
    for p in poison:
        assert bool(torch.isnan(p).all())


def test_k_worker_step_over_a_stack_of_blocks(sdp, orc):
    """K workers, L blocks, each worker holding p of them (block-level forward masking): every worker runs the stack
    (skipped blocks are identities), writes the gradients of the blocks it holds into its row of a block-granular
    buffer, and the coverage average divides each block by the number of workers that hold it."""
    K, L, p = 3, 4, 3
    Bt, S, d, H, hd, F = 1, 24, 32, 2, 8, 48
    E = H * hd
    rows = (3 * E + E + 3 * F)  # parameter rows of one block, each d long
    mask, idx, pos, cov = sdp.make_masks(K, L, p, 77, True)
    want_mask = orc.make_masks(K, L, p, 77, True)
    assert (mask.cpu().numpy() == want_mask).all()
    blocks = [_setup(500 + l, Bt, S, d, H, hd, F, "f32") for l in range(L)]
    bufs = [torch.full((L, rows * d), float("nan"), device="cuda") for _ in range(K)]
    refs = [np.zeros((L, rows * d)) for _ in range(K)]
    for k in range(K):
        print(f"  worker {k}: blocks {np.flatnonzero(want_mask[k]).tolist()}", flush=True)
        x = blocks[0]["X"].cuda() * (1 + k)
        dy = blocks[0]["dY"].cuda()
        xs, saves = [x], []
        for l in range(L):
            c = {n: v.cuda() for n, v in blocks[l].items()}
            y, saved = sdp.block_fwd("fm", int(want_mask[k][l]), Bt, S, hd, xs[-1], c["Wqkv"], c["WoT"], c["W1"], c["W3"], c["W2T"])
            xs.append(y); saves.append(saved)
        g = dy
        for l in reversed(range(L)):
            c = {n: v.cuda() for n, v in blocks[l].items()}
            g, grads = sdp.block_bwd("fm", int(want_mask[k][l]), Bt, S, hd, xs[l], g, c["Wqkv"], c["WoT"], c["W1"], c["W3"], c["W2T"], saves[l])
            if grads is not None:
                bufs[k][l] = torch.cat([t.reshape(-1) for t in grads])
        torch.cuda.synchronize()
        # the oracle's chain
        rx = [_f64(blocks[0]["X"]) * (1 + k)]
        for l in range(L):
            r = orc.block_step("fm", int(want_mask[k][l]), Bt, S, hd, rx[-1], np.zeros_like(rx[-1]), *_oracle_weights(blocks[l]))
            rx.append(r["Y"])
        rg = _f64(blocks[0]["dY"])
        for l in reversed(range(L)):
            r = orc.block_step("fm", int(want_mask[k][l]), Bt, S, hd, rx[l], rg, *_oracle_weights(blocks[l]))
            rg = r["dX"]
            refs[k][l] = np.concatenate([r[n].reshape(-1) for n in ("dWq", "dWk", "dWv", "dWoT", "dW1", "dW3", "dW2T")])
        assert_close(xs[-1].cpu().numpy(), rx[-1], 1e-4, f"worker {k} output of the stack")
        assert_close(g.cpu().numpy(), rg, 1e-4, f"worker {k} gradient below the stack")
        held = np.flatnonzero(want_mask[k])
        assert_close(bufs[k][torch.from_numpy(held).cuda()].cpu().numpy(), refs[k][held], 1e-4, f"worker {k} block gradients")
    avg, c = sdp.coverage_grad_avg(bufs, mask)
    torch.cuda.synchronize()
    want, wc = orc.gated_average(refs, want_mask)
    assert (c.cpu().numpy() == wc).all() and (wc >= 1).all()
    assert_close(avg.cpu().numpy(), want, 1e-4, "coverage average over blocks")


def _filled(shape, dtype, fill):
    t = torch.empty(shape, dtype=dtype, device="cuda")
    t.view(torch.uint8).fill_({"zero": 0, "nan": 0xFF, "big": 0x46}[fill])
    return t


@pytest.mark.parametrize("mode,m,rule", [("fm", 1, "through"), ("bm", 0, "through")])
def test_results_do_not_depend_on_what_workspace_and_outputs_held(sdp, mode, m, rule):
    """Nothing uninitialised is read: workspaces and output buffers pre-filled with NaN patterns, or with large
    finite values, give the same bits as zeroed ones."""
    Bt, S, d, H, hd, F = 2, 200, 256, 4, 64, 520
    t = {n: v.cuda() for n, v in _setup(70, Bt, S, d, H, hd, F, "bf16").items()}
    X, dY, Wqkv, WoT, W1, W3, W2T = (t[n] for n in ("X", "dY", "Wqkv", "WoT", "W1", "W3", "W2T"))
    dt, T, E = X.dtype, Bt * S, H * hd
    Es = H * sdp.attn_saved_head_width(dt, hd)
    res = {}
    for fill in ("zero", "nan", "big"):
        wsf = _filled((sdp.block_fwd_workspace_bytes(dt, Bt, S, d, H, hd, F) + 256,), torch.uint8, fill)
        wsb = _filled((sdp.block_bwd_workspace_bytes(dt, Bt, S, d, H, hd, F) + 256,), torch.uint8, fill)
        fo = (_filled((T, d), dt, fill), _filled((T, d), dt, fill), _filled((T, 3 * Es), dt, fill), _filled((T, Es), dt, fill),
              _filled((Bt, H, S), torch.float32, fill), _filled((T, F), dt, fill), _filled((T, F), dt, fill))
        Y, saved = sdp.block_fwd(mode, m, Bt, S, hd, X, Wqkv, WoT, W1, W3, W2T, out=fo, ws=wsf)
        bo = (_filled((T, d), dt, fill),)
        if m:
            bo += (_filled((3, E, d), dt, fill), _filled((E, d), dt, fill)) + tuple(_filled((F, d), dt, fill) for _ in range(3))
        dX, grads = sdp.block_bwd(mode, m, Bt, S, hd, X, dY, Wqkv, WoT, W1, W3, W2T, saved, dx_rule=rule, out=bo, ws=wsb)
        torch.cuda.synchronize()
        res[fill] = [t.clone().view(torch.uint8) for t in (Y,) + tuple(saved) + (dX,) + (tuple(grads) if grads else ())]
    for fill in ("nan", "big"):
        assert len(res[fill]) == len(res["zero"])
        for i, (a, b) in enumerate(zip(res["zero"], res[fill])):
            assert torch.equal(a, b), f"block {mode} m={m}: tensor {i} depends on the previous contents of a buffer ({fill})"
