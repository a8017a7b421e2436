"""GPU parity of the head-masked attention block (forward and backward) against the fp64 oracle.

Every output element is compared; tolerance 2e-2 for bf16 inputs with fp32 accumulation (metric in
helpers.err_report).  Head masks come from the library's sampler at head granularity and are checked bit for
bit against the oracle's.
"""
import numpy as np
import pytest
import torch

import workloads
import rounding_model as rm
from helpers import assert_close, assert_close_rows, assert_close_with_model
from workloads import AttnWorkload

pytestmark = pytest.mark.gpu

TOL = 2e-2
TOL_F32 = 1e-5
# Weight gradients behind the attention core pass through two more bf16 roundings than the MLP's (the
# probabilities and the logit gradients are MFMA operands) on top of those of dO, dQ/dK/dV and the result; the
# relative error per element then has a standard deviation near 0.4 % of the tensor's rms (the normwise
# figure), and the largest of 10^5 - 10^6 elements lies 4.5 - 5.5 deviations out.  The benchmark spec's bound of
# 2e-2 is kept for the normwise error; the elementwise maximum gets 3e-2.
TOL_ELEM_DW = 3e-2


@pytest.fixture(scope="module")
def sdp():
    import paper_2507_09029_amd as m

    assert torch.cuda.is_available()
    m.lib()
    return m


def held_rows(heads, hd):
    return np.concatenate([np.arange(h * hd, (h + 1) * hd) for h in heads])


def run_case(sdp, orc, w, workers, dw_layout="compact", mode="fm"):
    tol = TOL_F32 if w.dtype == "f32" else TOL
    tol_dw = None if w.dtype == "f32" else TOL_ELEM_DW
    Wqkv, WoT = workloads.attn_weights(w)
    dWqkv, dWoT = Wqkv.cuda(), WoT.cuda()
    mask, idx, pos, cov = sdp.make_masks(w.K, w.H, w.ph, w.mask_seed, True)
    want_mask = orc.make_masks(w.K, w.H, w.ph, w.mask_seed, True)
    assert (mask.cpu().numpy() == want_mask).all()
    W64 = [workloads.to_f64(Wqkv[i]) for i in range(3)] + [workloads.to_f64(WoT)]
    E_all = w.H * w.hd
    for k in workers:
        print(f"  {w.name} worker {k} {mode} {w.dtype} Bt={w.Bt} S={w.S} d={w.d} H={w.H} hd={w.hd} ph={w.ph} {dw_layout}", flush=True)
        X, dY = workloads.attn_batch(w, k)
        heads = np.flatnonzero(want_mask[k])
        assert (idx[k].cpu().numpy() == heads).all()
        Y, QKV, O, LSE = sdp.masked_attn_fwd(mode, w.Bt, w.S, w.hd, X.cuda(), dWqkv, dWoT, idx[k])
        out = None
        if dw_layout == "scatter":
            out = (torch.empty((w.T, w.d), dtype=X.dtype, device="cuda"),
                   torch.full((3, E_all, w.d), float("nan"), dtype=X.dtype, device="cuda"),
                   torch.full((E_all, w.d), float("nan"), dtype=X.dtype, device="cuda"))
        dX, gWqkv, gWoT = sdp.masked_attn_bwd(mode, w.Bt, w.S, w.hd, X.cuda(), dY.cuda(), dWqkv, dWoT, idx[k], QKV, O, LSE,
                                              dw_layout=dw_layout, out=out)
        torch.cuda.synchronize()
        ref = orc.attn_worker_step(w.Bt, w.S, w.hd, want_mask[k], workloads.to_f64(X), workloads.to_f64(dY), *W64, mode=mode)
        assert ref["nonzero_off_mask"] == 0
        held = held_rows(heads, w.hd)
        # heads the forward pass and the core ran on: the held ones, or all of them under backward masking
        rows = held if mode == "fm" else np.arange(E_all)
        E = rows.size
        # per-token tensors: one scale per row (a token's output averages over all earlier tokens, so the row
        # norms fall with the position); weight gradients: one scale per tensor
        assert_close_rows(workloads.to_f64(Y), ref["Y"], tol, "Y")
        # narrow bf16 heads are saved padded to 64 columns: the padding must hold exact zeros
        hw = sdp.attn_saved_head_width(QKV.dtype, w.hd)
        if hw != w.hd:
            assert not bool(QKV.reshape(w.T, -1, hw)[:, :, w.hd:].any()) and not bool(O.reshape(w.T, -1, hw)[:, :, w.hd:].any())
        got_qkv = workloads.to_f64(sdp.attn_unpad(QKV, w.hd))
        for i, name in enumerate("QKV"):
            assert_close_rows(got_qkv[:, i * E:(i + 1) * E], ref[name][:, rows], tol, name)
        assert_close_rows(workloads.to_f64(sdp.attn_unpad(O, w.hd)), ref["O"][:, rows], tol, "O")
        # base-2 log-sum-exp of the scaled logits, from the oracle's Q and K
        q = ref["Q"][:, rows].reshape(w.Bt, w.S, -1, w.hd)
        kk = ref["K"][:, rows].reshape(w.Bt, w.S, -1, w.hd)
        z = np.einsum("bshr,buhr->bhsu", q, kk) / np.sqrt(w.hd)
        z = np.where(np.tril(np.ones((w.S, w.S), bool)), z, -np.inf)
        zmax = z.max(axis=-1, keepdims=True)
        lse2 = (zmax[..., 0] + np.log(np.exp(z - zmax).sum(axis=-1))) / np.log(2.0)
        assert np.abs(LSE.cpu().numpy() - lse2).max() <= tol * max(1.0, np.abs(lse2).max())
        assert_close_rows(workloads.to_f64(dX), ref["dX"], tol, "dX")
        g = workloads.to_f64(gWqkv)
        go = workloads.to_f64(gWoT)
        if dw_layout == "scatter":
            off = np.setdiff1d(np.arange(E_all), held)
            assert np.isnan(g[:, off]).all() and np.isnan(go[off]).all(), "rows of heads not held must stay untouched"
            g, go = g[:, held], go[held]
        rows = held  # weight gradients exist for the held heads only, in both regimes
        model = None
        if w.dtype == "bf16" and w.S > 1:
            # the same arithmetic with only the bf16 rounding points: the kernels' weight gradients may be no further
            # from the oracle than this puts them (see helpers.assert_close_with_model)
            model = rm.attn_model(w.Bt, w.S, w.hd, want_mask[k], workloads.to_f64(X), workloads.to_f64(dY), *W64, mode=mode)
        for i, name in enumerate(("dWq", "dWk", "dWv")):
            if w.S == 1 and i < 2:
                # a softmax over one key is constant: the exact gradient is zero, and what is left of the
                # cancellation dP - delta in fp32 must be negligible next to the other gradients
                assert not ref[name].any()
                assert np.abs(g[i]).max() <= 1e-5 * np.sqrt(np.mean(ref["dWv"][rows] ** 2))
                continue
            if model is not None:
                assert_close_with_model(g[i], model[name][rows], ref[name][rows], tol, name, elem_allow=tol_dw)
            else:
                assert_close(g[i], ref[name][rows], tol, name, elem_tol=tol_dw)
        if model is not None:
            assert_close_with_model(go, model["dWoT"][rows], ref["dWoT"][rows], tol, "dWoT", elem_allow=tol_dw)
        else:
            assert_close(go, ref["dWoT"][rows], tol, "dWoT", elem_tol=tol_dw)


CASES = [
    AttnWorkload("one_tile", 1, 64, 64, 2, 64, 1, 2, 31),
    AttnWorkload("one_token", 3, 1, 64, 2, 64, 2, 2, 32),
    AttnWorkload("two_heads_of_four", 2, 128, 128, 4, 64, 2, 4, 33),
    AttnWorkload("ragged_seq_all_heads", 2, 200, 136, 3, 64, 3, 2, 34),     # C = 1: the dense block; S % 64 = 8
    AttnWorkload("ragged_depth", 1, 300, 72, 4, 64, 1, 4, 35),             # d % 16 != 0: plain contraction kernels
    AttnWorkload("several_blocks", 2, 520, 256, 8, 64, 4, 4, 36),          # 5 query blocks, tail of 8
    AttnWorkload("odd_tokens", 1, 77, 64, 2, 64, 1, 2, 37),                # T % 8 != 0
    # plain core: fp32 (1e-5), the paper's head width 50, bf16 with head widths other than 64
    AttnWorkload("f32_hd64", 2, 150, 96, 4, 64, 2, 4, 38, "f32"),
    AttnWorkload("f32_hd50_odd_sizes", 2, 93, 75, 3, 50, 2, 2, 39, "f32"),
    AttnWorkload("f32_hd128", 1, 70, 64, 2, 128, 1, 2, 40, "f32"),
    AttnWorkload("bf16_hd32", 2, 130, 128, 4, 32, 2, 4, 42),               # padded to 64: MFMA core
    AttnWorkload("bf16_hd96", 1, 100, 72, 3, 96, 2, 2, 43),
    # the paper's 500M / 1B head width (hidden 1200 / 24 heads, 1600 / 32 heads): bf16 heads of 50 padded to 64
    AttnWorkload("bf16_hd50", 2, 200, 200, 4, 50, 2, 4, 44),
    AttnWorkload("bf16_hd50_all_heads_odd", 1, 333, 104, 3, 50, 3, 2, 45),
    AttnWorkload("bf16_hd50_paper_500M_width", 1, 256, 1200, 24, 50, 12, 4, 46),
]


@pytest.mark.parametrize("w", CASES, ids=[w.name for w in CASES])
def test_attention_all_outputs(sdp, orc, w):
    run_case(sdp, orc, w, range(min(w.K, 2)))


def test_scatter_layout_leaves_other_heads_alone(sdp, orc):
    run_case(sdp, orc, CASES[2], [1], dw_layout="scatter")
    run_case(sdp, orc, CASES[5], [0], dw_layout="scatter", mode="bm")
    run_case(sdp, orc, CASES[12], [1], dw_layout="scatter")            # padded heads: the padding rows go nowhere
    run_case(sdp, orc, CASES[12], [0], dw_layout="scatter", mode="bm")


def test_padded_heads_backward_masking(sdp, orc):
    run_case(sdp, orc, CASES[12], [0, 1], mode="bm")
    run_case(sdp, orc, CASES[13], [0], mode="bm")


BM_CASES = [CASES[0], CASES[2], CASES[3], CASES[4], CASES[5], CASES[6], CASES[7], CASES[8], CASES[10]]


@pytest.mark.parametrize("w", BM_CASES, ids=[w.name for w in BM_CASES])
def test_attention_backward_masking_all_outputs(sdp, orc, w):
    """Dense forward and dX, weight gradients on the held heads only."""
    run_case(sdp, orc, w, range(min(w.K, 2)), mode="bm")


def test_argument_errors(sdp):
    w = CASES[2]
    Wqkv, WoT = (t.cuda() for t in workloads.attn_weights(w))
    X, _ = workloads.attn_batch(w, 0)
    idx = torch.tensor([0, 2], dtype=torch.int32, device="cuda")
    with pytest.raises(sdp.SdpError):  # bf16 heads wider than 64 are not padded: rows must be multiples of 16 bytes (3 x 84 = 252 rows)
        sdp.masked_attn_fwd("fm", w.Bt, w.S, 84, X.cuda(), Wqkv[:, :252].contiguous(), WoT[:252].contiguous(), idx)
    with pytest.raises(sdp.SdpError):  # more held heads than heads
        sdp.masked_attn_fwd("fm", w.Bt, w.S, w.hd, X.cuda(), Wqkv, WoT, torch.arange(5, dtype=torch.int32, device="cuda"))


def test_attention_full_step_average(sdp, orc):
    """Whole N-SDP step at head granularity: head masks -> K workers' forward + backward (scatter layout into
    full-size gradient buffers) -> coverage-normalised average with one mask byte per parameter row."""
    from helpers import err_report

    w = AttnWorkload("step", 2, 96, 128, 8, 64, 4, 4, 41)
    Wqkv, WoT = workloads.attn_weights(w)
    dWqkv, dWoT = Wqkv.cuda(), WoT.cuda()
    W64 = [workloads.to_f64(Wqkv[i]) for i in range(3)] + [workloads.to_f64(WoT)]
    mask, idx, pos, cov = sdp.make_masks(w.K, w.H, w.ph, w.mask_seed, True)
    want_mask = orc.make_masks(w.K, w.H, w.ph, w.mask_seed, True)
    assert (mask.cpu().numpy() == want_mask).all()
    E_all = w.H * w.hd
    bufs = [torch.full((4 * E_all, w.d), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in range(w.K)]
    refs = []
    for k in range(w.K):
        X, dY = workloads.attn_batch(w, k)
        Y, QKV, O, LSE = sdp.masked_attn_fwd("fm", w.Bt, w.S, w.hd, X.cuda(), dWqkv, dWoT, idx[k])
        out = (torch.empty((w.T, w.d), dtype=X.dtype, device="cuda"), bufs[k][: 3 * E_all].view(3, E_all, w.d), bufs[k][3 * E_all:])
        sdp.masked_attn_bwd("fm", w.Bt, w.S, w.hd, X.cuda(), dY.cuda(), dWqkv, dWoT, idx[k], QKV, O, LSE, dw_layout="scatter", out=out)
        r = orc.attn_worker_step(w.Bt, w.S, w.hd, want_mask[k], workloads.to_f64(X), workloads.to_f64(dY), *W64)
        refs.append(np.concatenate([r["dWq"], r["dWk"], r["dWv"], r["dWoT"]]))
    # head h owns rows h hd .. of each of the four matrices
    row_mask_host = np.tile(np.repeat(want_mask, w.hd, axis=1), (1, 4))
    row_mask = mask.repeat_interleave(w.hd, dim=1).repeat(1, 4).contiguous()
    assert (row_mask.cpu().numpy() == row_mask_host).all()
    avg, c = sdp.coverage_grad_avg(bufs, row_mask)
    torch.cuda.synchronize()
    host = [workloads.bf16_bits(b) for b in bufs]
    same_in, wc = orc.gated_average(host, row_mask_host)
    assert (c.cpu().numpy() == wc).all() and wc.min() >= 1
    assert_close(avg.cpu().numpy(), same_in, 1e-5, "average of the GPU's gradients")
    want, _ = orc.gated_average(refs, row_mask_host)
    assert err_report(avg.cpu().numpy(), want)[1] <= TOL, "averaged gradient, normwise"


@pytest.mark.parametrize("mode", ["fm", "bm"])
def test_plain_core_and_mfma_core_agree_on_the_same_inputs(sdp, mode):
    """The same bf16-valued inputs through the fp32 path (plain contractions and plain attention core, no
    intermediate rounding) and through the bf16 path (MFMA contractions and MFMA core): two implementations that
    share no kernel must agree to the bf16 path's rounding, without the oracle in between."""
    from helpers import err_report, err_report_rows

    w = AttnWorkload("paths", 2, 320, 128, 4, 64, 2, 2, 44)
    Wqkv, WoT = workloads.attn_weights(w)
    X, dY = workloads.attn_batch(w, 0)
    mask, idx, pos, cov = sdp.make_masks(w.K, w.H, w.ph, w.mask_seed, True)
    outs = {}
    for name, conv in (("bf16", lambda t: t.cuda()), ("f32", lambda t: t.float().cuda())):
        Y, QKV, O, LSE = sdp.masked_attn_fwd(mode, w.Bt, w.S, w.hd, conv(X), conv(Wqkv), conv(WoT), idx[0])
        dX, gWqkv, gWoT = sdp.masked_attn_bwd(mode, w.Bt, w.S, w.hd, conv(X), conv(dY), conv(Wqkv), conv(WoT), idx[0], QKV, O, LSE)
        torch.cuda.synchronize()
        outs[name] = [workloads.to_f64(t) for t in (Y, O, dX)] + [workloads.to_f64(gWqkv).reshape(-1, w.d), workloads.to_f64(gWoT),
                                                                 LSE.double().cpu().numpy().reshape(-1, w.S)]
    for got, ref, what in zip(outs["bf16"], outs["f32"], ("Y", "O", "dX", "dWqkv", "dWoT", "LSE")):
        elem, norm = (err_report if what.startswith("dW") else err_report_rows)(got, ref)
        assert norm <= 1e-2 and elem <= 3e-2, f"{what}: elementwise {elem:.3e}, normwise {norm:.3e}"


def test_forward_core_with_logits_that_keep_growing(sdp, orc):
    """Keys later in a sequence carry larger logits, so a query's running maximum climbs far beyond what it was
    after the first tile: the forward kernel has to move its reference exponent (and rescale what it has
    accumulated) several times on the way.  The core is isolated from the projections: the oracle evaluates
    the attention of the Q, K, V the library stored (bf16 values, widened exactly), through selector matrices."""
    w = AttnWorkload("growing_logits", 2, 520, 128, 2, 64, 2, 2, 45)
    Wqkv, WoT = workloads.attn_weights(w)
    Wqkv = Wqkv.clone()
    Wqkv[:2] *= 10.0  # W_Q, W_K
    X, _ = workloads.attn_batch(w, 0)
    ramp = 0.25 + 1.75 * torch.arange(w.S, dtype=torch.float32) / (w.S - 1)  # token norm grows 8-fold along a sequence
    X = (X.float().view(w.Bt, w.S, w.d) * ramp[None, :, None]).view(w.T, w.d).to(X.dtype)
    heads = torch.arange(w.H, dtype=torch.int32, device="cuda")
    Y, QKV, O, LSE = sdp.masked_attn_fwd("fm", w.Bt, w.S, w.hd, X.cuda(), Wqkv.cuda(), WoT.cuda(), heads)
    torch.cuda.synchronize()
    E = w.H * w.hd
    qkv = workloads.to_f64(QKV)
    sel = [np.zeros((E, 3 * E)) for _ in range(3)]
    for i in range(3):
        sel[i][np.arange(E), i * E + np.arange(E)] = 1.0
    ref = orc.attn_fwd(w.Bt, w.S, w.hd, qkv, sel[0], sel[1], sel[2], np.zeros((E, 3 * E)))  # the output projection is not used
    assert (ref["Q"] == qkv[:, :E]).all() and (ref["V"] == qkv[:, 2 * E:]).all()
    q = ref["Q"].reshape(w.Bt, w.S, w.H, w.hd)
    k = ref["K"].reshape(w.Bt, w.S, w.H, w.hd)
    z = np.einsum("bshr,buhr->bhsu", q, k) / np.sqrt(w.hd) / np.log(2.0)
    z = np.where(np.tril(np.ones((w.S, w.S), bool)), z, -np.inf)
    # the case does what it is meant to: maxima over the first 64 keys against maxima over all keys
    growth = z.max(axis=-1)[..., 64:] - z[..., :64].max(axis=-1)[..., 64:]
    assert np.median(growth) > 16.0, f"median growth of the running maximum {np.median(growth):.1f}"
    zmax = z.max(axis=-1, keepdims=True)
    lse2 = zmax[..., 0] + np.log2(np.exp2(z - zmax).sum(axis=-1))
    assert np.abs(LSE.cpu().numpy() - lse2).max() <= 1e-4 * np.abs(lse2).max()
    assert_close_rows(workloads.to_f64(O), ref["O"], TOL, "O")


def _filled(shape, dtype, fill):
    t = torch.empty(shape, dtype=dtype, device="cuda")
    t.view(torch.uint8).fill_({"zero": 0, "nan": 0xFF, "big": 0x46}[fill])
    return t


POISON = [w for w in CASES if w.name in ("two_heads_of_four", "ragged_depth", "several_blocks", "bf16_hd50", "f32_hd50_odd_sizes")]


@pytest.mark.parametrize("mode", ["fm", "bm"])
@pytest.mark.parametrize("w", POISON, ids=[w.name for w in POISON])
def test_results_do_not_depend_on_what_workspace_and_outputs_held(sdp, w, mode):
    """Nothing uninitialised is read: workspaces and output buffers pre-filled with NaN patterns, or with large
    finite values, give the same bits as zeroed ones (the padding columns of the saved tensors included)."""
    Wqkv, WoT = (t.cuda() for t in workloads.attn_weights(w))
    mask, idx, pos, cov = sdp.make_masks(w.K, w.H, w.ph, w.mask_seed, True)
    k = w.K - 1
    X, dY = (t.cuda() for t in workloads.attn_batch(w, k))
    dt = X.dtype
    n = w.ph if mode == "fm" else w.H
    hw = sdp.attn_saved_head_width(dt, w.hd)
    E = w.ph * w.hd
    res = {}
    for fill in ("zero", "nan", "big"):
        wsf = _filled((sdp.masked_attn_fwd_workspace_bytes(mode, dt, w.Bt, w.S, w.d, w.H, w.hd, w.ph) + 256,), torch.uint8, fill)
        wsb = _filled((sdp.masked_attn_bwd_workspace_bytes(mode, dt, w.Bt, w.S, w.d, w.H, w.hd, w.ph) + 256,), torch.uint8, fill)
        fo = (_filled((w.T, w.d), dt, fill), _filled((w.T, 3 * n * hw), dt, fill), _filled((w.T, n * hw), dt, fill),
              _filled((w.Bt, n, w.S), torch.float32, fill))
        Y, QKV, O, LSE = sdp.masked_attn_fwd(mode, w.Bt, w.S, w.hd, X, Wqkv, WoT, idx[k], out=fo, ws=wsf)
        bo = (_filled((w.T, w.d), dt, fill), _filled((3, E, w.d), dt, fill), _filled((E, w.d), dt, fill))
        back = sdp.masked_attn_bwd(mode, w.Bt, w.S, w.hd, X, dY, Wqkv, WoT, idx[k], QKV, O, LSE, out=bo, ws=wsb)
        torch.cuda.synchronize()
        res[fill] = [t.clone().view(torch.uint8) for t in (Y, QKV, O, LSE) + tuple(back)]
    for fill in ("nan", "big"):
        for name, a, b in zip(("Y", "QKV", "O", "LSE", "dX", "dWqkv", "dWoT"), res["zero"], res[fill]):
            assert torch.equal(a, b), f"{w.name} {mode}: {name} depends on the previous contents of a buffer ({fill})"
