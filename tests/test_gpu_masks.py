"""GPU parity, bit-exact: mask matrix, gather indices, ranks and coverage counts against the oracle."""
import numpy as np
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sdp():
    import paper_2507_09029_amd as m

    assert torch.cuda.is_available(), "these tests need the GPU"
    m.lib()
    return m


CASES = [
    (workloads.CONFIG1.K, workloads.CONFIG1.F, workloads.CONFIG1.p, workloads.CONFIG1.mask_seed, True),
    (workloads.CONFIG2.K, workloads.CONFIG2.F, workloads.CONFIG2.p, workloads.CONFIG2.mask_seed, True),
    (workloads.CONFIG3.K, workloads.CONFIG3.F, workloads.CONFIG3.p, workloads.CONFIG3.mask_seed, True),
    (workloads.CONFIG5.K, workloads.CONFIG5.R, workloads.CONFIG5.p, workloads.CONFIG5.mask_seed, False),
    (1, 1, 1, 3, True), (3, 7, 3, 4, True), (8, 2049, 300, 5, False), (64, 4097, 4097, 6, True), (2, 2048, 1024, 7, True),
]


@pytest.mark.parametrize("K,F,p,seed,cover", CASES)
def test_make_masks_matches_oracle(sdp, orc, K, F, p, seed, cover):
    print(f"make_masks K={K} F={F} p={p} seed={seed} cover={cover}", flush=True)
    mask, idx, pos, cov = sdp.make_masks(K, F, p, seed, cover)
    torch.cuda.synchronize()
    want_mask = orc.make_masks(K, F, p, seed, cover)
    widx, wpos, wcount, wcov = orc.index_masks(want_mask, idx_ld=p)
    assert (mask.cpu().numpy() == want_mask).all()
    assert (idx.cpu().numpy() == widx).all()
    assert (pos.cpu().numpy() == wpos).all()
    assert (cov.cpu().numpy() == wcov).all()
    assert (wcount == p).all()


@pytest.mark.parametrize("K,F,p,seed", [
    (workloads.CONFIG2.K, workloads.CONFIG2.F, workloads.CONFIG2.p, 31), (workloads.CONFIG3.K, workloads.CONFIG3.F, workloads.CONFIG3.p, 32),
    (3, 100, 41, 33), (6, 2049, 300, 34),
])
def test_make_masks_balanced_matches_oracle(sdp, orc, K, F, p, seed):
    print(f"make_masks balanced K={K} F={F} p={p} seed={seed}", flush=True)
    mask, idx, pos, cov = sdp.make_masks(K, F, p, seed, "balanced")
    torch.cuda.synchronize()
    want_mask = orc.make_masks_balanced(K, F, p, seed)
    widx, wpos, wcount, wcov = orc.index_masks(want_mask, idx_ld=p)
    assert (mask.cpu().numpy() == want_mask).all()
    assert (idx.cpu().numpy() == widx).all()
    assert (pos.cpu().numpy() == wpos).all()
    assert (cov.cpu().numpy() == wcov).all()
    assert (wcount == p).all()


@pytest.mark.parametrize("K,F,density,idx_ld", [
    (5, 333, 0.4, 333), (8, 2048, 0.5, 2048), (3, 2049, 0.9, 100), (1, 6000, 0.01, 6000), (8, 100000, 0.69, 100000),
])
def test_index_masks_general_masks(sdp, orc, K, F, density, idx_ld):
    print(f"index_masks K={K} F={F} density={density} idx_ld={idx_ld}", flush=True)
    rng = np.random.default_rng(K * 1000 + F)
    m = (rng.random((K, F)) < density).astype(np.uint8)
    m[0] = 0                    # a worker with nothing
    if K > 1:
        m[1] = 1                # a worker with everything
    if K > 2:
        m[2] *= 7               # any non-zero byte counts as 1
    idx, pos, count, cov = sdp.index_masks(torch.from_numpy(m).cuda(), idx_ld=idx_ld)
    torch.cuda.synchronize()
    widx, wpos, wcount, wcov = orc.index_masks(m, idx_ld=idx_ld)
    assert (count.cpu().numpy() == wcount).all()
    assert (idx.cpu().numpy() == widx).all()
    assert (pos.cpu().numpy() == wpos).all()
    assert (cov.cpu().numpy() == wcov).all()


@pytest.mark.parametrize("K,F,p,seed,cover", [
    (workloads.CONFIG2.K, workloads.CONFIG2.F, workloads.CONFIG2.p, workloads.CONFIG2.mask_seed, True),
    (workloads.CONFIG5.K, workloads.CONFIG5.R, workloads.CONFIG5.p, workloads.CONFIG5.mask_seed, False),
    (4, 4096, 2048, 9, "balanced"), (1, 1, 1, 3, True), (64, 4097, 1000, 6, False), (3, 100001, 20000, 8, False),
])
def test_mask_rho2_matches_oracle(sdp, orc, K, F, p, seed, cover):
    """Distance to uniform masking (Thm. 3.1): integer load histogram bit-exact, the value to fp64 rounding."""
    print(f"mask_rho2 K={K} F={F} p={p} seed={seed} cover={cover}", flush=True)
    mask, _, _, cov = sdp.make_masks(K, F, p, seed, cover)
    rho2, hist = sdp.mask_rho2(K, cov)
    want_mask = orc.make_masks_balanced(K, F, p, seed) if cover == "balanced" else orc.make_masks(K, F, p, seed, cover)
    want = orc.rho2(want_mask)
    loads = np.bincount(want_mask.sum(axis=0, dtype=np.int64), minlength=65)
    assert (hist.cpu().numpy() == loads).all()
    # the oracle adds K F non-negative terms one after the other (error at most K F ulps of the sum); the library
    # adds at most K + 1 products of exact counts
    assert abs(rho2 - want) <= (K * F + 64) * 2.0 ** -52 * max(1.0, abs(want))
    if cover == "balanced":  # K p a multiple of F: every load is K p / F
        assert abs(rho2 - F * (F / (K * p) - 1 / K)) < 1e-9


def test_mask_rho2_rejects_loads_above_K(sdp):
    cov = torch.full((1000,), 5, dtype=torch.uint8, device="cuda")
    with pytest.raises(RuntimeError):
        sdp.mask_rho2(4, cov)
    rho2, hist = sdp.mask_rho2(5, cov)  # all five workers hold everything
    assert rho2 == 0.0 and int(hist[5]) == 1000


def test_mask_rho2_rejects_loads_above_the_largest_K(sdp):
    """With K = 64 (the largest accepted) a count byte above 64 must still be an error, not load 64."""
    cov = torch.full((4096,), 64, dtype=torch.uint8, device="cuda")
    rho2, hist = sdp.mask_rho2(64, cov)
    assert rho2 == 0.0 and int(hist[64]) == 4096
    cov[1234] = 200
    with pytest.raises(RuntimeError):
        sdp.mask_rho2(64, cov)
