"""GPU parity of the coverage-normalised gradient average against the oracle (fp64)."""
import numpy as np
import pytest
import torch

import workloads
from helpers import assert_close

pytestmark = pytest.mark.gpu

TOL_SUM = 1e-5  # fp32 sum of at most 64 terms and one division, against fp64


@pytest.fixture(scope="module")
def sdp():
    import paper_2507_09029_amd as m

    assert torch.cuda.is_available()
    m.lib()
    return m


def _np_inputs(grads):
    if grads[0].dtype == torch.bfloat16:
        return [workloads.bf16_bits(g) for g in grads]
    return [g.cpu().numpy() for g in grads]


@pytest.mark.parametrize("K,R,D,p,dtype", [
    (4, 300, 256, 150, "bf16"), (8, 1000, 2048, 690, "bf16"), (8, 257, 1536, 100, "f32"), (3, 50, 520, 20, "bf16"),
    (2, 64, 8, 32, "f32"), (5, 40, 7, 20, "bf16"), (5, 40, 13, 20, "f32"), (1, 10, 512, 4, "bf16"), (64, 33, 1024, 3, "bf16"),
    (8, 3072, 256, 1536, "f32"),
])
def test_avg_matches_oracle_with_poisoned_off_mask_rows(sdp, orc, K, R, D, p, dtype):
    print(f"avg K={K} R={R} D={D} p={p} {dtype}", flush=True)
    mask = orc.make_masks(K, R, p, 77, False)
    tmask = torch.from_numpy(mask)
    grads = workloads.grad_buffers(K, R, D, 1e-3, dtype, poison_mask=tmask)
    dev = [g.cuda() for g in grads]
    out, cov = sdp.coverage_grad_avg(dev, tmask.cuda())
    torch.cuda.synchronize()
    want, wcov = orc.gated_average(_np_inputs(grads), mask)
    assert (cov.cpu().numpy() == wcov).all()                       # counts: bit exact
    got = out.cpu().numpy()
    assert np.isfinite(got).all()                                  # NaN in uncovered rows was never read
    assert (got[wcov == 0] == 0.0).all()                           # nobody covers the row: 0, not NaN
    assert_close(got, want, TOL_SUM, "avg")
    # the clean run gives the same bits
    clean = workloads.grad_buffers(K, R, D, 1e-3, dtype)
    out2, _ = sdp.coverage_grad_avg([g.cuda() for g in clean], tmask.cuda())
    assert torch.equal(out2, out)


def test_avg_block_level_masks(sdp, orc):
    """Block-level subnetworks (Sec. 3.2: a worker keeps or skips whole blocks): the same average with one mask
    byte per block, a row being all the parameters of a block.  32 blocks of 2^20 parameters, 22 kept per worker
    (the paper's 1B setting keeps 22 of 32 blocks), 8 workers."""
    K, R, D, p = 8, 32, 1 << 20, 22
    mask = orc.make_masks(K, R, p, 91, True)
    tmask = torch.from_numpy(mask)
    print(f"avg block-level K={K} blocks={R} D={D} p={p}", flush=True)
    grads = workloads.grad_buffers(K, R, D, 1e-3, "bf16", device="cuda", poison_mask=tmask)
    out, cov = sdp.coverage_grad_avg(grads, tmask.cuda())
    torch.cuda.synchronize()
    want, wcov = orc.gated_average([workloads.bf16_bits(g) for g in grads], mask)
    assert (cov.cpu().numpy() == wcov).all() and (wcov >= 1).all()
    assert_close(out.cpu().numpy(), want, TOL_SUM, "block-level avg")


def test_avg_full_coverage_is_the_mean_and_single_worker_is_identity(sdp):
    K, R, D = 8, 100, 1024
    grads = [g.cuda() for g in workloads.grad_buffers(K, R, D, 1.0, "f32")]
    ones = torch.ones((K, R), dtype=torch.uint8, device="cuda")
    out, cov = sdp.coverage_grad_avg(grads, ones)
    ref = torch.stack([g.double() for g in grads]).mean(0)
    assert (cov == K).all()
    assert_close(out.cpu().numpy(), ref.cpu().numpy(), TOL_SUM, "mean")
    out1, cov1 = sdp.coverage_grad_avg(grads[:1], ones[:1].contiguous())
    assert torch.equal(out1, grads[0]) and (cov1 == 1).all()


def test_avg_empty_input_and_binding_errors(sdp):
    g = [torch.empty((0, 64), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    out, cov = sdp.coverage_grad_avg(g, torch.empty((2, 0), dtype=torch.uint8, device="cuda"))
    assert out.shape == (0, 64) and cov.shape == (0,)
    with pytest.raises(sdp.SdpError):
        sdp.coverage_grad_avg([], torch.empty((0, 0), dtype=torch.uint8, device="cuda"))


@pytest.mark.parametrize("K,R,D,p,dtype", [
    (4, 300, 256, 150, "bf16"), (8, 1000, 2048, 690, "bf16"), (8, 257, 1536, 100, "f32"), (5, 40, 13, 20, "f32"),
    (5, 40, 7, 20, "bf16"), (1, 10, 512, 4, "bf16"), (8, 40000, 512, 27600, "bf16"),
    (20, 700, 1032, 90, "bf16"), (64, 33, 1024, 3, "f32"),  # more workers than one batch of mask bytes
])
def test_squared_norm_of_the_average_matches_oracle(sdp, orc, K, R, D, p, dtype):
    """sdp_coverage_grad_sqnorm against the oracle's fp64 sum; NaN in rows nobody covers is never read; the value
    equals the norm of what sdp_coverage_grad_avg stores (same fp32 averages), and repeats bit for bit."""
    print(f"sqnorm K={K} R={R} D={D} p={p} {dtype}", flush=True)
    mask = orc.make_masks(K, R, p, 78, False)
    tmask = torch.from_numpy(mask)
    grads = workloads.grad_buffers(K, R, D, 1e-3, dtype, poison_mask=tmask)
    dev = [g.cuda() for g in grads]
    got = sdp.coverage_grad_sqnorm(dev, tmask.cuda())
    again = sdp.coverage_grad_sqnorm(dev, tmask.cuda())
    avg, _ = sdp.coverage_grad_avg(dev, tmask.cuda())
    torch.cuda.synchronize()
    want = orc.gated_average_sqnorm(_np_inputs(grads), mask)
    got = float(got.cpu()[0])
    assert np.isfinite(got) and got == float(again.cpu()[0])
    assert abs(got - want) <= 1e-5 * want  # fp32 averages (relative error 1e-7 each), fp64 sum
    stored = float((avg.double() ** 2).sum().cpu())
    assert abs(got - stored) <= 1e-12 * stored


def test_squared_norm_empty_and_errors(sdp):
    import ctypes

    L = sdp.lib()
    out = torch.full((1,), 7.0, dtype=torch.float64, device="cuda")
    ws = torch.empty(4096, dtype=torch.uint8, device="cuda")
    ptrs = (ctypes.c_void_p * 2)(None, None)
    assert L.sdp_coverage_grad_sqnorm(2, 0, 16, 1, ptrs, None, out.data_ptr(), ws.data_ptr(), ws.numel(), None) == 0
    torch.cuda.synchronize()
    assert float(out.cpu()[0]) == 0.0
    g = torch.zeros((4, 16), dtype=torch.bfloat16, device="cuda")
    m = torch.ones((2, 4), dtype=torch.uint8, device="cuda")
    with pytest.raises(RuntimeError):
        sdp.coverage_grad_sqnorm([g, g], m, ws=torch.empty(16, dtype=torch.uint8, device="cuda")[:0])


def test_hbm_streaming_probe_copies_and_reports_a_rate(sdp):
    """The measurement aid: the copy form really copies (whole 16 KiB chunks), both forms report a positive rate."""
    src = torch.randint(0, 255, (3 * 16384 + 100,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    assert sdp.probe_hbm_gbs(src, dst, launches=2) > 0
    assert torch.equal(dst[: 3 * 16384], src[: 3 * 16384]) and int(dst[3 * 16384:].sum()) == 0
    assert sdp.probe_hbm_gbs(src, launches=2) > 0
