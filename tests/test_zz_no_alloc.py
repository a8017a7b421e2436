"""GPU test of sdp_index_masks_static, the entry point for callers that cannot allocate: its chunk-count table is
a fixed array of the library.  Two calls in a row on one GPU, the second on a smaller input, each checked bit
for bit against sdp_index_masks (workspace from the caller) and against the oracle."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sdp():
    import paper_2507_09029_amd as m

    assert torch.cuda.is_available(), "these tests need the GPU"
    m.lib()
    return m


def _mask(K, F, density, seed):
    rng = np.random.default_rng(seed)
    m = (rng.random((K, F)) < density).astype(np.uint8)
    m[0, : F // 3] = 0
    if K > 1:
        m[1] = 1
    return m


def _check(sdp, orc, m, idx_ld):
    K, F = m.shape
    mask = torch.from_numpy(m).cuda()
    out = (torch.full((K, idx_ld), -7, dtype=torch.int32, device="cuda"), torch.full((K, F), -7, dtype=torch.int32, device="cuda"),
           torch.full((K,), -7, dtype=torch.int32, device="cuda"), torch.full((F,), 99, dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    got = sdp.index_masks_static(mask, idx_ld=idx_ld, out=out)
    assert torch.cuda.memory_allocated() == before  # nothing was taken from torch's allocator either
    torch.cuda.synchronize()
    ref = sdp.index_masks(mask, idx_ld=idx_ld)
    torch.cuda.synchronize()
    want = orc.index_masks(m, idx_ld=idx_ld)
    for name, g, r, w in zip(("idx", "pos", "count", "cov"), got, ref, want):
        assert torch.equal(g, r), f"{name}: static variant differs from sdp_index_masks"
        assert (g.cpu().numpy() == w).all(), f"{name}: differs from the oracle"


def test_index_masks_static_two_calls_second_smaller(sdp, orc):
    print("index_masks_static: K=8 F=488282 then K=5 F=70001 then a short row", flush=True)
    _check(sdp, orc, _mask(8, 488282, 0.69, 1), 488282)   # 239 chunks per row: the table is used
    _check(sdp, orc, _mask(5, 70001, 0.4, 2), 30000)      # smaller, ragged, idx rows cut short: stale counts must not leak
    _check(sdp, orc, _mask(3, 3000, 0.5, 3), 3000)        # short rows: the single-launch route, no table


def test_index_masks_static_rejects_sizes_beyond_its_table(sdp):
    L = sdp.lib()
    fake = ctypes.c_void_p(0x1000)
    F = 2048 * 1025  # 1025 chunks x 64 workers = 65600 counts > 65536
    assert L.sdp_index_masks_static(64, F, fake, fake, F, fake, fake, fake, None) == -2
    assert L.sdp_index_masks_static(4, 100, None, fake, 100, fake, fake, fake, None) == -1
