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
