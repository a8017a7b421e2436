"""The device-side path under HIP graph capture: a worker's compaction, forward, backward and the coverage
average are captured once and replayed several times with new inputs, with eager work and synchronisations
between the replays; every replay must reproduce the eager result bit for bit (the kernels are deterministic).
The library records no memset nodes on this path (sdp_make_masks, which samples on the host, is not part of it).
"""
import pytest
import torch

import workloads
from workloads import AttnWorkload, MlpWorkload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sdp():
    import paper_2507_09029_amd as m

    assert torch.cuda.is_available()
    m.lib()
    return m


def _replay_against_eager(run, inputs, variants, outputs):
    """run() reads the static `inputs` and writes the static `outputs`; variants = list of input tuples."""
    def load(v):
        for dst, src in zip(inputs, v):
            dst.copy_(src)

    refs = []
    for v in variants:  # eager references (also performs every first-launch set-up before the capture)
        load(v)
        run()
        torch.cuda.synchronize()
        refs.append([o.clone() for o in outputs])
    graph = torch.cuda.CUDAGraph()
    cap = torch.cuda.Stream()
    cap.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(cap):
        with torch.cuda.graph(graph, stream=cap):
            run()
    torch.cuda.synchronize()
    for rep in (0, 1, 0, 1, 1):
        load(variants[rep])
        for o in outputs:
            o.fill_(float("nan")) if o.is_floating_point() else o.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(outputs, refs[rep]):
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), f"replay of variant {rep} differs from the eager run"
        # the program's own eager work between replays
        load(variants[1 - rep])
        run()
        torch.cuda.synchronize()


def test_mlp_step_replays_like_eager(sdp):
    w = MlpWorkload("graph_bf16_fm", "bf16", 512, 256, 1024, 512, 2, "fm", 51)
    Wd = [t.cuda() for t in workloads.mlp_weights(w)]
    mask, idx0, pos0, cov0 = sdp.make_masks(w.K, w.F, w.p, w.mask_seed, True)
    batches = [tuple(t.cuda() for t in workloads.mlp_batch(w, k)) for k in range(2)]
    X, dY = (torch.empty_like(t) for t in batches[0])
    other = torch.randn((3 * w.F, w.d), device="cuda").to(torch.bfloat16)  # the second worker's gradient buffer
    buf = torch.zeros((3 * w.F, w.d), dtype=torch.bfloat16, device="cuda")
    Y = torch.empty((w.T, w.d), dtype=torch.bfloat16, device="cuda")
    G = torch.empty((w.T, w.p), dtype=torch.bfloat16, device="cuda")
    U = torch.empty_like(G)
    dX = torch.empty_like(Y)
    avg = torch.empty((3 * w.F, w.d), dtype=torch.float32, device="cuda")
    cov = torch.empty((3 * w.F,), dtype=torch.uint8, device="cuda")
    row_mask = mask.repeat(1, 3).contiguous()
    ws_i = torch.empty(sdp.index_masks_workspace_bytes(w.K, w.F), dtype=torch.uint8, device="cuda")
    ws_f = torch.empty(sdp.masked_mlp_fwd_workspace_bytes("fm", X.dtype, w.T, w.d, w.F, w.p), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(sdp.masked_mlp_bwd_workspace_bytes("fm", X.dtype, w.T, w.d, w.F, w.p), dtype=torch.uint8, device="cuda")
    idx_holder = {}

    def run():
        idx, pos, count, c = sdp.index_masks(mask, idx_ld=w.p, ws=ws_i)
        idx_holder["idx"] = idx
        sdp.masked_mlp_fwd("fm", X, *Wd, idx[0], out=(Y, G, U), ws=ws_f)
        sdp.masked_mlp_bwd("fm", X, dY, *Wd, idx[0], G, U, dw_layout="scatter",
                           out=(dX, buf[: w.F], buf[w.F: 2 * w.F], buf[2 * w.F:]), ws=ws_b)
        sdp.coverage_grad_avg([buf, other], row_mask, out=avg, cov=cov)

    _replay_against_eager(run, (X, dY), batches, (Y, dX, avg))
    assert torch.equal(idx_holder["idx"], idx0)


def test_attention_step_replays_like_eager(sdp):
    w = AttnWorkload("graph_attn", 2, 192, 128, 4, 64, 2, 2, 52)
    Wqkv, WoT = (t.cuda() for t in workloads.attn_weights(w))
    mask, idx, pos, cov = sdp.make_masks(w.K, w.H, w.ph, w.mask_seed, True)
    batches = [tuple(t.cuda() for t in workloads.attn_batch(w, k)) for k in range(2)]
    X, dY = (torch.empty_like(t) for t in batches[0])
    E = w.ph * w.hd
    bf = dict(dtype=torch.bfloat16, device="cuda")
    fo = (torch.empty((w.T, w.d), **bf), torch.empty((w.T, 3 * E), **bf), torch.empty((w.T, E), **bf),
          torch.empty((w.Bt, w.ph, w.S), dtype=torch.float32, device="cuda"))
    bo = (torch.empty((w.T, w.d), **bf), torch.empty((3, E, w.d), **bf), torch.empty((E, w.d), **bf))
    ws_f = torch.empty(sdp.masked_attn_fwd_workspace_bytes("fm", X.dtype, w.Bt, w.S, w.d, w.H, w.hd, w.ph), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(sdp.masked_attn_bwd_workspace_bytes("fm", X.dtype, w.Bt, w.S, w.d, w.H, w.hd, w.ph), dtype=torch.uint8, device="cuda")

    def run():
        Y, QKV, O, LSE = sdp.masked_attn_fwd("fm", w.Bt, w.S, w.hd, X, Wqkv, WoT, idx[0], out=fo, ws=ws_f)
        sdp.masked_attn_bwd("fm", w.Bt, w.S, w.hd, X, dY, Wqkv, WoT, idx[0], QKV, O, LSE, out=bo, ws=ws_b)

    _replay_against_eager(run, (X, dY), batches, (fo[0], bo[0], bo[1], bo[2]))
