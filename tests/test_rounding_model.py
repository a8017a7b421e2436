"""The rounding model of the bf16 path (tests/rounding_model.py) against the oracle.

With the roundings switched off the model IS the oracle's arithmetic by another route (torch matmuls instead of
C loops): it must agree with the oracle to fp64 rounding, which ties the model to the pinned oracle.  With the
roundings on, its distance from the oracle is the error that storing and multiplying bf16 values causes by itself;
the figures asserted here are the basis of the elementwise allowances in the GPU tests (the GPU tests also compare
the kernels with this model directly, at a tighter bound than with the oracle)."""
import numpy as np
import pytest

import rounding_model as rm
import workloads
from helpers import err_report
from workloads import AttnWorkload, MlpWorkload


def _bf16_inputs(*arrays):
    import torch

    return [rm.rb(torch.as_tensor(a)).numpy() for a in arrays]


def _mlp_case(w, k, orc):
    W = [workloads.to_f64(t) for t in workloads.mlp_weights(w)]
    X, dY = (workloads.to_f64(t) for t in workloads.mlp_batch(w, k))
    mask = orc.make_masks(w.K, w.F, w.p, w.mask_seed, True)
    return mask[k], X, dY, W


@pytest.mark.parametrize("mode", ["fm", "bm"])
def test_mlp_model_without_rounding_is_the_oracle(orc, mode):
    w = MlpWorkload("m", "bf16", 96, 40, 64, 24, 3, mode, 5)
    mk, X, dY, W = _mlp_case(w, 1, orc)
    ref = orc.worker_step(mode, mk, X, dY, *W)
    got = rm.mlp_model(mode, mk, X, dY, *W, on=False)
    for n in ("Y", "dX", "dW1", "dW3", "dW2T"):
        np.testing.assert_allclose(got[n], ref[n], rtol=1e-10, atol=1e-12, err_msg=n)
    run = np.flatnonzero(mk) if mode == "fm" else np.arange(w.F)
    np.testing.assert_allclose(got["G"][:, run], ref["G"][:, run], rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("mode", ["fm", "bm"])
def test_attention_model_without_rounding_is_the_oracle(orc, mode):
    w = AttnWorkload("a", 2, 37, 24, 3, 8, 2, 2, 5)
    Wqkv, WoT = workloads.attn_weights(w)
    X, dY = (workloads.to_f64(t) for t in workloads.attn_batch(w, 0))
    Wl = [workloads.to_f64(Wqkv[i]) * 10 for i in range(3)] + [workloads.to_f64(WoT) * 10]
    hm = orc.make_masks(w.K, w.H, w.ph, w.mask_seed, True)[0]
    ref = orc.attn_worker_step(w.Bt, w.S, w.hd, hm, X, dY, *Wl, mode=mode)
    got = rm.attn_model(w.Bt, w.S, w.hd, hm, X, dY, *Wl, mode=mode, on=False)
    for n in ("Q", "K", "V", "O", "Y", "dX", "dWq", "dWk", "dWv", "dWoT"):
        np.testing.assert_allclose(got[n], ref[n], rtol=1e-9, atol=1e-11, err_msg=n)


@pytest.mark.parametrize("mode,m,rule", [("fm", 1, "through"), ("fm", 0, "through"), ("bm", 0, "through"), ("bm", 0, "skip")])
def test_block_model_without_rounding_is_the_oracle(orc, mode, m, rule):
    rng = np.random.default_rng(3)
    Bt, S, d, H, hd, F = 2, 19, 12, 2, 4, 20
    X, dY = rng.standard_normal((Bt * S, d)), rng.standard_normal((Bt * S, d))
    W = [rng.standard_normal((H * hd, d)) * 0.3 for _ in range(4)] + [rng.standard_normal((F, d)) * 0.3 for _ in range(3)]
    ref = orc.block_step(mode, m, Bt, S, hd, X, dY, *W, dx_rule=rule)
    got = rm.block_model(mode, m, Bt, S, hd, X, dY, *W, dx_rule=rule, on=False)
    for n in ("Y", "dX", "dWq", "dWk", "dWv", "dWoT", "dW1", "dW3", "dW2T"):
        np.testing.assert_allclose(got[n], ref[n], rtol=1e-9, atol=1e-11, err_msg=n)


def test_mlp_rounding_alone_stays_below_the_stated_tolerance_at_benchmark_like_sizes(orc):
    """512 tokens, the smallest bf16 parity shape: the bf16 roundings alone put the weight gradients 1.2e-2 - 2.0e-2
    (elementwise) and 3e-3 (normwise) from the exact result; per-token tensors up to 1.8e-2 (elementwise) and 3e-3 (normwise)."""
    w = MlpWorkload("m", "bf16", 512, 256, 1024, 512, 4, "fm", 3)
    mk, X, dY, W = _mlp_case(w, 3, orc)
    ref = orc.worker_step("fm", mk, X, dY, *W)
    got = rm.mlp_model("fm", mk, X, dY, *W)
    S = np.flatnonzero(mk)
    for n in ("dW1", "dW3", "dW2T"):
        e, nrm = err_report(got[n][S], ref[n][S])
        assert 5e-3 < e < 2e-2 and nrm < 5e-3, (n, e, nrm)
    for n in ("Y", "dX"):
        e, nrm = err_report(got[n], ref[n])
        assert e < 2e-2 and nrm < 5e-3, (n, e, nrm)


def test_weight_gradients_over_few_tokens_exceed_the_stated_tolerance_by_rounding_alone(orc):
    """A weight-gradient entry that sums over a few dozen tokens keeps most of its operands' rounding error: at 40
    tokens the model alone is 2e-2 - 4e-2 (elementwise) from the exact result while the normwise error stays at a few
    1e-3.  This is why the seeded random small shapes allow 4e-2 elementwise for the bf16 weight gradients."""
    worst = 0.0
    for seed in range(6):
        w = MlpWorkload("m", "bf16", 40, 64, 128, 64, 2, "fm", 20 + seed)
        mk, X, dY, W = _mlp_case(w, 0, orc)
        ref = orc.worker_step("fm", mk, X, dY, *W)
        got = rm.mlp_model("fm", mk, X, dY, *W)
        S = np.flatnonzero(mk)
        for n in ("dW1", "dW3", "dW2T"):
            e, nrm = err_report(got[n][S], ref[n][S])
            assert nrm < 1e-2 and e < 4e-2, (n, e, nrm)
            worst = max(worst, e)
    assert worst > 1.5e-2


def test_attention_rounding_alone_reaches_the_elementwise_allowance(orc):
    """Attention weight gradients pass two more bf16 roundings (probabilities and logit gradients as matrix
    operands): at 2 x 256 tokens the roundings alone put them 1.3e-2 - 3e-2 elementwise from the exact result,
    a few 1e-3 normwise.  The GPU tests allow 3e-2 elementwise for these four tensors."""
    w = AttnWorkload("a", 2, 256, 256, 4, 64, 2, 2, 11)
    Wqkv, WoT = workloads.attn_weights(w)
    X, dY = (workloads.to_f64(t) for t in workloads.attn_batch(w, 0))
    Wl = [workloads.to_f64(Wqkv[i]) for i in range(3)] + [workloads.to_f64(WoT)]
    hm = orc.make_masks(w.K, w.H, w.ph, w.mask_seed, True)[0]
    ref = orc.attn_worker_step(w.Bt, w.S, w.hd, hm, X, dY, *Wl)
    got = rm.attn_model(w.Bt, w.S, w.hd, hm, X, dY, *Wl)
    rows = np.concatenate([np.arange(h * w.hd, (h + 1) * w.hd) for h in np.flatnonzero(hm)])
    worst = 0.0
    for n in ("dWq", "dWk", "dWv", "dWoT"):
        e, nrm = err_report(got[n][rows], ref[n][rows])
        print(n, e, nrm)
        assert e < 3e-2 and nrm < 1e-2, (n, e, nrm)
        worst = max(worst, e)
    assert worst > 1e-2
