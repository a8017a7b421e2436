"""GPU parity of the coverage average fused with AdamW against the oracle (fp64)."""
import numpy as np
import pytest
import torch

import workloads
from helpers import assert_close

pytestmark = pytest.mark.gpu

HP = dict(lr=4e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
TOL = 1e-5  # fp32 arithmetic (a sum of at most 64 terms, a division, a square root) against fp64


@pytest.fixture(scope="module")
def sdp():
    import paper_2507_09029_amd as m

    assert torch.cuda.is_available()
    m.lib()
    return m


def _state(R, D, seed):
    g = torch.Generator().manual_seed(seed)
    theta = torch.randn((R, D), generator=g) * 0.02
    m = torch.randn((R, D), generator=g) * 1e-4
    v = (torch.randn((R, D), generator=g) * 1e-4) ** 2
    return theta, m, v


@pytest.mark.parametrize("K,R,D,p,dtype,step", [
    (4, 300, 256, 150, "bf16", 1), (8, 1000, 2048, 690, "bf16", 7), (8, 257, 1536, 100, "f32", 1000), (3, 50, 520, 20, "bf16", 2),
    (5, 40, 7, 20, "bf16", 3), (5, 40, 13, 20, "f32", 3), (1, 10, 512, 4, "bf16", 1), (64, 33, 1024, 3, "bf16", 50),
])
def test_adamw_matches_oracle(sdp, orc, K, R, D, p, dtype, step):
    print(f"avg+adamw K={K} R={R} D={D} p={p} {dtype} step={step}", flush=True)
    mask = orc.make_masks(K, R, p, 77, False)
    tmask = torch.from_numpy(mask)
    grads = workloads.grad_buffers(K, R, D, 1e-3, dtype, poison_mask=tmask)
    theta, m, v = _state(R, D, 5)
    dth, dm, dv = theta.cuda(), m.cuda(), v.cuda()
    lowp = torch.full((R, D), 7.0, dtype=torch.bfloat16, device="cuda")
    cov = sdp.coverage_avg_adamw([g.cuda() for g in grads], tmask.cuda(), dth, dm, dv, step=step, grad_scale=0.5,
                                 theta_bf16=lowp, **HP)
    torch.cuda.synchronize()
    g_np = [workloads.bf16_bits(g) for g in grads] if dtype == "bf16" else [g.numpy() for g in grads]
    wth, wm, wv, wcov = orc.avg_adamw(g_np, mask, theta.numpy(), m.numpy(), v.numpy(), step=step, grad_scale=0.5, **HP)
    assert (cov.cpu().numpy() == wcov).all()
    got_th, got_m, got_v = dth.cpu().numpy(), dm.cpu().numpy(), dv.cpu().numpy()
    assert np.isfinite(got_th).all() and np.isfinite(got_m).all() and np.isfinite(got_v).all()
    off = wcov == 0
    # rows nobody covers: bit-identical state, bf16 copy not written
    assert (got_th[off] == theta.numpy()[off]).all() and (got_m[off] == m.numpy()[off]).all() and (got_v[off] == v.numpy()[off]).all()
    assert (lowp.cpu().float().numpy()[off] == 7.0).all()
    assert_close(got_m, wm, TOL, "m")
    assert_close(got_v, wv, TOL, "v")
    assert_close(got_th, wth, TOL, "theta")
    # the update itself (theta moves by about lr per step, far above fp32 resolution of theta)
    assert_close(got_th.astype(np.float64) - theta.numpy(), wth - theta.numpy(), 1e-4, "theta update")
    # the bf16 copy is the updated fp32 value rounded to nearest even
    on = ~off
    assert torch.equal(lowp.cpu()[torch.from_numpy(on)], dth.cpu()[torch.from_numpy(on)].to(torch.bfloat16))


def test_adamw_argument_errors(sdp):
    g = [torch.zeros((4, 8), dtype=torch.bfloat16, device="cuda")]
    mask = torch.ones((1, 4), dtype=torch.uint8, device="cuda")
    th, m, v = (torch.zeros((4, 8), device="cuda") for _ in range(3))
    for bad in (dict(HP, beta1=1.0), dict(HP, eps=0.0), dict(HP, lr=-1.0)):
        with pytest.raises(sdp.SdpError):
            sdp.coverage_avg_adamw(g, mask, th, m, v, step=1, **bad)
    with pytest.raises(sdp.SdpError):
        sdp.coverage_avg_adamw(g, mask, th, m, v, step=0, **HP)


@pytest.mark.parametrize("max_norm,gscale", [(1.0, 30.0), (1.0, 1e-3)])
def test_clipped_update_on_the_device_matches_oracle(sdp, orc, max_norm, gscale):
    """Global-norm clipping without a round trip to the host: squared norms of two parameter groups ->
    sdp_clip_scale -> the fused update reads the coefficient from device memory.  Gradient scale 30 puts the
    norm far above the threshold (coefficient < 1), 1e-3 far below (coefficient 1)."""
    K, D = 4, 256
    groups = []
    for gi, (R, p) in enumerate(((300, 150), (77, 40))):
        mask = orc.make_masks(K, R, p, 90 + gi, False)
        grads = workloads.grad_buffers(K, R, D, gscale, "bf16", poison_mask=torch.from_numpy(mask))
        groups.append((R, mask, grads))
    sq = torch.zeros((2,), dtype=torch.float64, device="cuda")
    for gi, (R, mask, grads) in enumerate(groups):
        sdp.coverage_grad_sqnorm([g.cuda() for g in grads], torch.from_numpy(mask).cuda(), out=sq[gi:gi + 1])
    scale = sdp.clip_scale(sq, max_norm)
    want_sq = [orc.gated_average_sqnorm([workloads.bf16_bits(g) for g in grads], mask) for R, mask, grads in groups]
    want_scale = orc.clip_scale(want_sq, max_norm)
    torch.cuda.synchronize()
    assert (want_scale < 0.5) == (gscale > 1.0) and (want_scale == 1.0) == (gscale < 1.0)
    assert abs(float(scale.cpu()[0]) - want_scale) <= 1e-5 * want_scale
    for gi, (R, mask, grads) in enumerate(groups):
        theta, m, v = _state(R, D, 11 + gi)
        dth, dm, dv = theta.cuda(), m.cuda(), v.cuda()
        sdp.coverage_avg_adamw([g.cuda() for g in grads], torch.from_numpy(mask).cuda(), dth, dm, dv, step=3,
                               grad_scale_dev=scale, **HP)
        torch.cuda.synchronize()
        wth, wm, wv, wcov = orc.avg_adamw([workloads.bf16_bits(g) for g in grads], mask, theta.numpy(), m.numpy(), v.numpy(),
                                          step=3, grad_scale=want_scale, **HP)
        assert_close(dm.cpu().numpy(), wm, TOL, "m")
        assert_close(dv.cpu().numpy(), wv, 2 * TOL, "v")  # the coefficient's own 1e-5 enters squared
        assert_close(dth.cpu().numpy(), wth, TOL, "theta")


def test_clip_scale_argument_errors(sdp):
    sq = torch.ones((2,), dtype=torch.float64, device="cuda")
    for bad in (0.0, -1.0, float("inf"), float("nan")):
        with pytest.raises(sdp.SdpError):
            sdp.clip_scale(sq, bad)
    with pytest.raises(sdp.SdpError):
        sdp.clip_scale(sq[:0], 1.0)
