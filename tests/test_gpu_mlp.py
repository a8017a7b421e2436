"""GPU parity of the masked SwiGLU MLP (forward and backward, both regimes) against the fp64 oracle.

Small and medium shapes: the oracle computes every output element.  Tolerances (metric in
helpers.err_report): 1e-5 for the fp32 path, 2e-2 for bf16 inputs with fp32 accumulation.
"""
import numpy as np
import pytest
import torch

import workloads
import rounding_model as rm
from helpers import assert_close, assert_close_with_model
from workloads import MlpWorkload

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


@pytest.fixture(scope="module")
def sdp():
    import paper_2507_09029_amd as m

    assert torch.cuda.is_available()
    m.lib()
    return m


def run_case(sdp, orc, w, workers, dw_layout="compact", dw_elem_tol=None):
    """dw_elem_tol: elementwise bound for the weight gradients when it differs from the tolerance (see
    test_gpu_random_shapes.py); the normwise bound is always the tolerance."""
    tol = TOL[w.dtype]
    W1, W3, W2T = workloads.mlp_weights(w)
    dW = [t.cuda() for t in (W1, W3, W2T)]
    mask, idx, pos, cov = sdp.make_masks(w.K, w.F, w.p, w.mask_seed, True)
    want_mask = orc.make_masks(w.K, w.F, w.p, w.mask_seed, True)
    assert (mask.cpu().numpy() == want_mask).all()
    W64 = [workloads.to_f64(t) for t in (W1, W3, W2T)]
    for k in workers:
        print(f"  {w.name} worker {k} {w.mode} {w.dtype} T={w.T} d={w.d} F={w.F} p={w.p} {dw_layout}", flush=True)
        X, dY = workloads.mlp_batch(w, k)
        Y, G, U = sdp.masked_mlp_fwd(w.mode, X.cuda(), *dW, idx[k])
        if dw_layout == "scatter":
            out = (torch.empty((w.T, w.d), dtype=X.dtype, device="cuda"),) + tuple(
                torch.full((w.F, w.d), float("nan"), dtype=X.dtype, device="cuda") for _ in range(3))
        else:
            out = None
        dX, dW1, dW3, dW2T = sdp.masked_mlp_bwd(w.mode, X.cuda(), dY.cuda(), *dW, idx[k], G, U, dw_layout=dw_layout, out=out)
        torch.cuda.synchronize()
        ref = orc.worker_step(w.mode, want_mask[k], workloads.to_f64(X), workloads.to_f64(dY), *W64)
        S = np.flatnonzero(want_mask[k])
        model = None
        assert ref["nonzero_off_mask"] == 0
        assert_close(workloads.to_f64(Y), ref["Y"], tol, "Y")
        assert_close(workloads.to_f64(dX), ref["dX"], tol, "dX")
        cols = S if w.mode == "fm" else slice(None)
        assert_close(workloads.to_f64(G), ref["G"][:, cols], tol, "G")
        assert_close(workloads.to_f64(U), ref["U"][:, cols], tol, "U")
        for name, got in (("dW1", dW1), ("dW3", dW3), ("dW2T", dW2T)):
            g64 = workloads.to_f64(got)
            if dw_layout == "scatter":
                off = np.flatnonzero(want_mask[k] == 0)
                assert np.isnan(g64[off]).all(), "rows off the mask must stay untouched"
                g64 = g64[S]
            if w.dtype == "bf16":
                # no further from the oracle than the bf16 rounding points alone put the result (see helpers)
                if model is None:
                    model = rm.mlp_model(w.mode, want_mask[k], workloads.to_f64(X), workloads.to_f64(dY), *W64)
                assert_close_with_model(g64, model[name][S], ref[name][S], tol, name, elem_allow=dw_elem_tol)
            else:
                assert_close(g64, ref[name][S], tol, name, elem_tol=dw_elem_tol)


SMALL = [
    MlpWorkload("tiny_f32_fm", "f32", 8, 8, 16, 8, 2, "fm", 11),
    MlpWorkload("ragged_f32_fm", "f32", 77, 40, 130, 37, 4, "fm", 12),
    MlpWorkload("ragged_f32_bm", "f32", 77, 40, 130, 37, 4, "bm", 12),
    MlpWorkload("full_cover_f32_fm", "f32", 64, 32, 64, 64, 2, "fm", 13),       # C = 1: the dense MLP
    MlpWorkload("tiles_bf16_fm", "bf16", 264, 136, 520, 264, 4, "fm", 14),      # several tiles + ragged tails
    MlpWorkload("tiles_bf16_bm", "bf16", 264, 136, 520, 264, 4, "bm", 14),
    MlpWorkload("tails16_bf16_fm", "bf16", 272, 144, 528, 272, 4, "fm", 18),    # MFMA path, every depth ends in a partial step
    MlpWorkload("tails16_bf16_bm", "bf16", 272, 144, 528, 304, 4, "bm", 18),
    MlpWorkload("tails48_bf16_fm", "bf16", 304, 176, 560, 240, 4, "fm", 19),    # depth tails of 48, ragged rows / columns
    MlpWorkload("aligned_bf16_fm", "bf16", 512, 256, 1024, 512, 4, "fm", 15),
    MlpWorkload("aligned_bf16_bm", "bf16", 512, 256, 1024, 768, 4, "bm", 16),
    MlpWorkload("full_cover_bf16_bm", "bf16", 256, 128, 256, 256, 2, "bm", 17),
    MlpWorkload("tiny_bf16_fm", "bf16", 8, 16, 32, 16, 2, "fm", 20),            # one MFMA tile, almost all of it out of range
    MlpWorkload("tiny_bf16_bm", "bf16", 16, 16, 48, 16, 3, "bm", 21),
    MlpWorkload("full_cover_bf16_fm", "bf16", 48, 64, 128, 128, 2, "fm", 22),   # C = 1 on the MFMA path
]


@pytest.mark.parametrize("w", SMALL, ids=[w.name for w in SMALL])
def test_small_shapes_all_outputs(sdp, orc, w):
    run_case(sdp, orc, w, range(min(w.K, 2)))


def test_config1_all_workers(sdp, orc):
    run_case(sdp, orc, workloads.CONFIG1, range(workloads.CONFIG1.K))


def test_scatter_layout_leaves_off_mask_rows_alone(sdp, orc):
    run_case(sdp, orc, SMALL[1], [0], dw_layout="scatter")
    run_case(sdp, orc, SMALL[5], [1], dw_layout="scatter")


def test_config1_full_step_average(sdp, orc):
    """Whole path at config 1: masks -> K workers' fwd+bwd (scatter layout) -> coverage average."""
    w = workloads.CONFIG1
    W1, W3, W2T = workloads.mlp_weights(w)
    dW = [t.cuda() for t in (W1, W3, W2T)]
    W64 = [workloads.to_f64(t) for t in (W1, W3, W2T)]
    mask, idx, pos, cov = sdp.make_masks(w.K, w.F, w.p, w.mask_seed, True)
    want_mask = orc.make_masks(w.K, w.F, w.p, w.mask_seed, True)
    bufs = [torch.full((3 * w.F, w.d), float("nan"), dtype=torch.float32, device="cuda") for _ in range(w.K)]
    ref_bufs = []
    for k in range(w.K):
        X, dY = workloads.mlp_batch(w, k)
        Y, G, U = sdp.masked_mlp_fwd("fm", X.cuda(), *dW, idx[k])
        out = (torch.empty((w.T, w.d), dtype=torch.float32, device="cuda"),
               bufs[k][0:w.F], bufs[k][w.F:2 * w.F], bufs[k][2 * w.F:])
        sdp.masked_mlp_bwd("fm", X.cuda(), dY.cuda(), *dW, idx[k], G, U, dw_layout="scatter", out=out)
        r = orc.worker_step("fm", want_mask[k], workloads.to_f64(X), workloads.to_f64(dY), *W64)
        ref_bufs.append(np.concatenate([r["dW1"], r["dW3"], r["dW2T"]]))
    row_mask = mask.repeat(1, 3).contiguous()  # neuron j owns row j of each of the three matrices
    avg, c = sdp.coverage_grad_avg(bufs, row_mask)
    torch.cuda.synchronize()
    want, wc = orc.gated_average(ref_bufs, np.tile(want_mask, (1, 3)))
    assert (c.cpu().numpy() == wc).all() and wc.min() >= 1
    assert_close(avg.cpu().numpy(), want, 1e-5, "averaged gradient")


@pytest.mark.parametrize("mode", ["fm", "bm"])
def test_fp32_path_and_bf16_path_agree_on_the_same_inputs(sdp, mode):
    """The same bf16-valued inputs through the fp32 kernels (plain FMA contractions, no intermediate rounding) and
    through the bf16 MFMA kernels: two implementations inside the library that share no contraction code must
    agree to the bf16 path's rounding (about 1e-2), without the oracle in between."""
    from helpers import err_report

    w = MlpWorkload("paths", "bf16", 512, 256, 1024, 512, 2, mode, 61)
    W = workloads.mlp_weights(w)
    X, dY = workloads.mlp_batch(w, 0)
    mask, idx, pos, cov = sdp.make_masks(w.K, w.F, w.p, w.mask_seed, True)
    outs = {}
    for name, conv in (("bf16", lambda t: t.cuda()), ("f32", lambda t: t.float().cuda())):
        Wd = [conv(t) for t in W]
        Y, G, U = sdp.masked_mlp_fwd(mode, conv(X), *Wd, idx[0])
        dX, dW1, dW3, dW2T = sdp.masked_mlp_bwd(mode, conv(X), conv(dY), *Wd, idx[0], G, U)
        torch.cuda.synchronize()
        outs[name] = [workloads.to_f64(t) for t in (Y, G, U, dX, dW1, dW3, dW2T)]
    for got, ref, what in zip(outs["bf16"], outs["f32"], ("Y", "G", "U", "dX", "dW1", "dW3", "dW2T")):
        elem, norm = err_report(got, ref)
        assert norm <= 1e-2 and elem <= 2e-2, f"{what}: elementwise {elem:.3e}, normwise {norm:.3e}"


def _filled(shape, dtype, fill):
    """A GPU tensor whose bytes are all zero, all 0xFF (NaN in bf16 and fp32) or all 0x46 (about 1.3e4 in both)."""
    t = torch.empty(shape, dtype=dtype, device="cuda")
    t.view(torch.uint8).fill_({"zero": 0, "nan": 0xFF, "big": 0x46}[fill])
    return t


POISON = [w for w in SMALL if w.name in ("ragged_f32_fm", "tiles_bf16_fm", "tiles_bf16_bm", "aligned_bf16_bm", "tiny_bf16_fm")] + [
    MlpWorkload("mixed_paths_bf16_fm", "bf16", 552, 440, 1536, 1312, 4, "fm", 23),  # depth 440: plain kernels beside MFMA ones
]


@pytest.mark.parametrize("w", POISON, ids=[w.name for w in POISON])
def test_results_do_not_depend_on_what_workspace_and_outputs_held(sdp, w):
    """Nothing uninitialised is read: the same calls with the workspaces and every output buffer pre-filled with
    NaN patterns, or with large finite values, give the bits they give over zeroed buffers."""
    Wd = [t.cuda() for t in workloads.mlp_weights(w)]
    mask, idx, pos, cov = sdp.make_masks(w.K, w.F, w.p, w.mask_seed, True)
    k = w.K - 1
    X, dY = (t.cuda() for t in workloads.mlp_batch(w, k))
    n = w.p if w.mode == "fm" else w.F
    res = {}
    for fill in ("zero", "nan", "big"):
        wsf = _filled((sdp.masked_mlp_fwd_workspace_bytes(w.mode, X.dtype, w.T, w.d, w.F, w.p) + 256,), torch.uint8, fill)
        wsb = _filled((sdp.masked_mlp_bwd_workspace_bytes(w.mode, X.dtype, w.T, w.d, w.F, w.p) + 256,), torch.uint8, fill)
        fo = (_filled((w.T, w.d), X.dtype, fill), _filled((w.T, n), X.dtype, fill), _filled((w.T, n), X.dtype, fill))
        Y, G, U = sdp.masked_mlp_fwd(w.mode, X, *Wd, idx[k], out=fo, ws=wsf)
        bo = (_filled((w.T, w.d), X.dtype, fill),) + tuple(_filled((w.p, w.d), X.dtype, fill) for _ in range(3))
        back = sdp.masked_mlp_bwd(w.mode, X, dY, *Wd, idx[k], G, U, out=bo, ws=wsb)
        torch.cuda.synchronize()
        res[fill] = [t.clone().view(torch.uint8) for t in (Y, G, U) + tuple(back)]
    for fill in ("nan", "big"):
        for name, a, b in zip(("Y", "G", "U", "dX", "dW1", "dW3", "dW2T"), res["zero"], res[fill]):
            assert torch.equal(a, b), f"{w.name}: {name} depends on the previous contents of a buffer ({fill})"
