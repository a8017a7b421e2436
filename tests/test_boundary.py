"""Host-only checks of the C-ABI library: it loads, exports everything include/*.h declares,
rejects bad arguments before launching anything, and its host mask sampler matches the oracle's
independent implementation of the same sampler bit for bit."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2507_09029_amd as sdp
from paper_2507_09029_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(0x1000)  # non-null, 16-byte aligned, never dereferenced: errors precede any launch


def declared_functions():
    import glob

    text = "".join(open(h).read() for h in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sdp_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = sdp.lib()
    names = declared_functions()
    assert {"sdp_make_masks", "sdp_masked_mlp_fwd", "sdp_masked_mlp_bwd", "sdp_coverage_grad_avg"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings():
    L = sdp.lib()
    seen = {L.sdp_status_string(s) for s in range(0, -7, -1)}
    assert len(seen) == 7 and L.sdp_status_string(-99) == b"unknown status"


def test_workspace_queries():
    assert sdp.index_masks_workspace_bytes(4, 1024) >= 4 * 1 * 4
    assert sdp.index_masks_workspace_bytes(8, 488282) >= 8 * 239 * 4
    assert sdp.index_masks_workspace_bytes(0, 10) == 0
    import torch
    fw = sdp.masked_mlp_fwd_workspace_bytes("fm", torch.bfloat16, 8192, 1536, 4096, 2048)
    assert fw >= 8192 * 2048 * 2
    bw = sdp.masked_mlp_bwd_workspace_bytes("bm", torch.bfloat16, 16384, 2048, 5504, 4128)
    assert bw >= 5 * 16384 * 5504 * 2
    assert sdp.masked_mlp_fwd_workspace_bytes("fm", torch.bfloat16, 8, 12, 16, 8) == 0  # d not a multiple of 8
    assert sdp.masked_mlp_fwd_workspace_bytes("fm", torch.float32, 8, 12, 16, 7) > 0


def test_argument_errors_are_caught_on_the_host():
    L = sdp.lib()
    big = ctypes.c_size_t(1 << 40)
    # make_masks
    assert L.sdp_make_masks(4, 16, 8, 1, 1, None, FAKE, FAKE, FAKE, FAKE, big, None) == -1
    assert L.sdp_make_masks(0, 16, 8, 1, 1, FAKE, FAKE, FAKE, FAKE, FAKE, big, None) == -1
    assert L.sdp_make_masks(65, 16, 8, 1, 1, FAKE, FAKE, FAKE, FAKE, FAKE, big, None) == -1
    assert L.sdp_make_masks(4, 16, 17, 1, 1, FAKE, FAKE, FAKE, FAKE, FAKE, big, None) == -2
    assert L.sdp_make_masks(2, 16, 7, 1, 1, FAKE, FAKE, FAKE, FAKE, FAKE, big, None) == -4
    assert L.sdp_make_masks(4, 16, 8, 1, 1, FAKE, FAKE, FAKE, FAKE, FAKE, ctypes.c_size_t(0), None) == -3
    assert L.sdp_make_masks(4, 16, 8, 1, 1, FAKE, FAKE, FAKE, FAKE, None, big, None) == -3
    # index_masks
    assert L.sdp_index_masks(4, 16, FAKE, FAKE, 17, FAKE, None, FAKE, FAKE, big, None) == -2
    assert L.sdp_index_masks(4, 16, FAKE, FAKE, 0, FAKE, None, FAKE, FAKE, big, None) == -2
    assert L.sdp_index_masks(4, 16, None, FAKE, 8, FAKE, None, FAKE, FAKE, big, None) == -1
    assert L.sdp_index_masks(4, 16, FAKE, FAKE, 8, FAKE, None, FAKE, FAKE, ctypes.c_size_t(8), None) == -3
    # rho^2
    out = ctypes.c_double(0.0)
    assert L.sdp_mask_rho2(4, 16, None, FAKE, ctypes.byref(out), None) == -1
    assert L.sdp_mask_rho2(4, 16, FAKE, None, ctypes.byref(out), None) == -1
    assert L.sdp_mask_rho2(4, 16, FAKE, FAKE, None, None) == -1
    assert L.sdp_mask_rho2(65, 16, FAKE, FAKE, ctypes.byref(out), None) == -1
    assert L.sdp_mask_rho2(4, 0, FAKE, FAKE, ctypes.byref(out), None) == -1
    assert L.sdp_mask_rho2(4, 1 << 31, FAKE, FAKE, ctypes.byref(out), None) == -2
    # squared norm of the average
    ptrs2 = (ctypes.c_void_p * 2)(FAKE, FAKE)
    assert sdp.lib().sdp_coverage_grad_sqnorm_workspace_bytes(488282, 2048) >= 8
    assert sdp.lib().sdp_coverage_grad_sqnorm_workspace_bytes(-1, 8) == 0
    assert L.sdp_coverage_grad_sqnorm(0, 4, 16, 1, ptrs2, FAKE, FAKE, FAKE, big, None) == -1
    assert L.sdp_coverage_grad_sqnorm(2, 4, 16, 3, ptrs2, FAKE, FAKE, FAKE, big, None) == -1
    assert L.sdp_coverage_grad_sqnorm(2, 4, 16, 1, ptrs2, None, FAKE, FAKE, big, None) == -1
    assert L.sdp_coverage_grad_sqnorm(2, 4, 16, 1, ptrs2, FAKE, None, FAKE, big, None) == -1
    assert L.sdp_coverage_grad_sqnorm(2, 1 << 38, 16, 1, ptrs2, FAKE, FAKE, FAKE, big, None) == -2
    assert L.sdp_coverage_grad_sqnorm(2, 4, 16, 1, ptrs2, FAKE, FAKE, None, big, None) == -3
    assert L.sdp_coverage_grad_sqnorm(2, 4, 16, 1, ptrs2, FAKE, FAKE, FAKE, ctypes.c_size_t(8), None) == -3
    # clip coefficient
    assert L.sdp_clip_scale(0, FAKE, ctypes.c_float(1.0), FAKE, None) == -1
    assert L.sdp_clip_scale(2, None, ctypes.c_float(1.0), FAKE, None) == -1
    assert L.sdp_clip_scale(2, FAKE, ctypes.c_float(1.0), None, None) == -1
    assert L.sdp_clip_scale(2, FAKE, ctypes.c_float(0.0), FAKE, None) == -1
    assert L.sdp_clip_scale(2, ctypes.c_void_p(0x1004), ctypes.c_float(1.0), FAKE, None) == -1
    # forward
    def fwd(mode=0, dt=1, T=16, d=16, F=32, p=16, X=FAKE, idx=FAKE, ws=FAKE, wsb=big):
        return L.sdp_masked_mlp_fwd(mode, dt, T, d, F, p, X, FAKE, FAKE, FAKE, idx, FAKE, FAKE, FAKE, ws, wsb, None)
    assert fwd(mode=2) == -1 and fwd(dt=5) == -1 and fwd(T=0) == -1 and fwd(X=None) == -1
    assert fwd(p=40) == -2 and fwd(p=0) == -2 and fwd(d=12) == -2 and fwd(p=12) == -2
    assert fwd(idx=None) == -1 and fwd(ws=None) == -3 and fwd(wsb=ctypes.c_size_t(16)) == -3
    assert fwd(X=ctypes.c_void_p(0x1004)) == -1  # misaligned
    # backward
    def bwd(mode=0, dt=1, T=16, d=16, F=32, p=16, dY=FAKE, lay=0, ws=FAKE, wsb=big):
        return L.sdp_masked_mlp_bwd(mode, dt, T, d, F, p, FAKE, dY, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                                    FAKE, lay, ws, wsb, None)
    assert bwd(mode=-1) == -1 and bwd(dY=None) == -1 and bwd(lay=2) == -1
    assert bwd(T=12) == -2 and bwd(p=33) == -2 and bwd(wsb=ctypes.c_size_t(1024)) == -3
    # average
    ptrs = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    assert L.sdp_coverage_grad_avg(0, 4, 8, 1, ptrs, FAKE, FAKE, FAKE, None) == -1
    hp = sdp.binding.AdamWParams(4e-3, 0.9, 0.95, 1e-8, 0.1, 1.0, 1)
    adam = lambda *a: L.sdp_coverage_avg_adamw(*a)
    assert adam(2, 4, 8, 1, ptrs, FAKE, FAKE, FAKE, FAKE, None, FAKE, None, None) == -1            # no hyper-parameters
    assert adam(2, 4, 8, 1, ptrs, FAKE, None, FAKE, FAKE, None, FAKE, ctypes.byref(hp), None) == -1  # no theta
    assert adam(0, 4, 8, 1, ptrs, FAKE, FAKE, FAKE, FAKE, None, FAKE, ctypes.byref(hp), None) == -1
    bad_hp = sdp.binding.AdamWParams(4e-3, 1.0, 0.95, 1e-8, 0.1, 1.0, 1)
    assert adam(2, 4, 8, 1, ptrs, FAKE, FAKE, FAKE, FAKE, None, FAKE, ctypes.byref(bad_hp), None) == -1
    assert adam(2, 0, 8, 1, ptrs, FAKE, FAKE, FAKE, FAKE, None, FAKE, ctypes.byref(hp), None) == 0   # nothing to do
    out = ctypes.c_double(0.0)
    assert L.sdp_probe_mfma_tflops(None, 4, 4, FAKE, ctypes.byref(out), None) == -1
    assert L.sdp_probe_mfma_tflops(FAKE, 0, 4, FAKE, ctypes.byref(out), None) == -1
    assert L.sdp_probe_mfma_operand_bytes() == 6 * 512 * 16 and L.sdp_probe_mfma_sink_bytes(2) == 2 * 512 * 4
    assert L.sdp_probe_hbm_gbs(0, None, FAKE, 1 << 20, 1, ctypes.byref(out), None) == -1
    assert L.sdp_probe_hbm_gbs(0, FAKE, FAKE, 1 << 20, 0, ctypes.byref(out), None) == -1
    assert L.sdp_probe_hbm_gbs(1, FAKE, FAKE, 1000, 1, ctypes.byref(out), None) == -1  # less than one chunk
    assert L.sdp_coverage_grad_avg(2, 4, 0, 1, ptrs, FAKE, FAKE, FAKE, None) == -1
    assert L.sdp_coverage_grad_avg(2, 4, 8, 7, ptrs, FAKE, FAKE, FAKE, None) == -1
    assert L.sdp_coverage_grad_avg(2, 4, 8, 1, None, FAKE, FAKE, FAKE, None) == -1
    assert L.sdp_coverage_grad_avg(2, -1, 8, 1, ptrs, FAKE, FAKE, FAKE, None) == -1
    bad = (ctypes.c_void_p * 2)(0x1000, 0)
    assert L.sdp_coverage_grad_avg(2, 4, 8, 1, bad, FAKE, FAKE, FAKE, None) == -1
    assert L.sdp_coverage_grad_avg(2, 4, 8, 1, ptrs, None, FAKE, FAKE, None) == -1
    assert L.sdp_coverage_grad_avg(2, 4, 8, 1, ptrs, FAKE, ctypes.c_void_p(0x1008), FAKE, None) == -1
    assert L.sdp_coverage_grad_avg(2, 0, 8, 1, ptrs, FAKE, FAKE, FAKE, None) == 0  # empty input: nothing to do


def test_binding_raises_sdp_error():
    with pytest.raises(sdp.SdpError) as e:
        sdp.sample_masks_host(2, 16, 7, 1, True)
    assert e.value.status == -4


@pytest.mark.parametrize("K,F,p,cover", [
    (4, 1024, 512, True), (4, 4096, 2048, True), (8, 5504, 4128, True), (8, 5504, 4128, False),
    (3, 7, 3, True), (2, 10, 5, True), (1, 5, 5, True), (8, 64, 8, True), (5, 33, 1, False), (8, 20000, 13800, False),
])
def test_host_sampler_matches_oracle_bit_for_bit(orc, K, F, p, cover):
    for seed in (20250709, 1, 2**63 + 12345):
        got = sdp.sample_masks_host(K, F, p, seed, cover).numpy()
        want = orc.make_masks(K, F, p, seed, cover)
        assert (got == want).all()


@pytest.mark.parametrize("K,F,p", [
    (4, 1024, 512), (4, 4096, 2048), (8, 5504, 4128), (3, 100, 41), (6, 97, 13), (5, 64, 64), (2, 50, 1), (3, 10, 0),
    (8, 688, 516), (1, 33, 7),
])
def test_balanced_sampler_matches_oracle_bit_for_bit(orc, K, F, p):
    # the library finds each weighted pick with a Fenwick tree, the oracle by a linear scan
    for seed in (20250709, 7, 2**63 + 12345):
        got = sdp.sample_masks_host(K, F, p, seed, "balanced").numpy()
        want = orc.make_masks_balanced(K, F, p, seed)
        assert (got == want).all()


def test_sampler_mode_is_validated():
    L = sdp.lib()
    buf = (ctypes.c_uint8 * 64)()
    assert L.sdp_sample_masks_host(2, 16, 8, 1, 3, buf) == -1
    assert L.sdp_sample_masks_host(2, 16, 8, 1, -1, buf) == -1
    assert L.sdp_sample_masks_host(2, 16, 4, 1, 2, buf) == 0  # balanced mode does not need K p >= F


def test_binding_module_does_not_touch_the_oracle():
    src = open(binding.__file__).read() + open(os.path.join(os.path.dirname(binding.__file__), "__init__.py")).read()
    assert "oracle" not in src


def test_attention_arguments_are_checked_on_the_host():
    import torch

    L = sdp.lib()
    big = ctypes.c_size_t(1 << 40)
    BF16, F32, FM, BM = 1, 0, 0, 1
    assert sdp.binding._DTYPES[torch.bfloat16] == BF16 and sdp.binding._DTYPES[torch.float32] == F32
    assert sdp.binding._MODES["fm"] == FM and sdp.binding._MODES["bm"] == BM
    ws = sdp.masked_attn_fwd_workspace_bytes("fm", torch.bfloat16, 4, 2048, 1536, 24, 64, 12)
    assert ws >= 4 * 768 * 4 + 1536 * 768 * 2
    wb = sdp.masked_attn_bwd_workspace_bytes("fm", torch.bfloat16, 4, 2048, 1536, 24, 64, 12)
    assert wb >= 8192 * 768 * 2 * (1 + 3 + 3 + 1) + 2 * 1536 * 8192 * 2
    # backward masking runs the core on all 24 heads: twice the activations of 12 held heads
    assert sdp.masked_attn_bwd_workspace_bytes("bm", torch.bfloat16, 4, 2048, 1536, 24, 64, 12) >= 8192 * 1536 * 2 * (1 + 3 + 3 + 1)
    assert sdp.masked_attn_fwd_workspace_bytes("fm", torch.float32, 4, 2048, 1536, 24, 64, 12) > ws   # fp32 elements
    assert sdp.masked_attn_fwd_workspace_bytes("fm", torch.float32, 4, 1024, 1200, 24, 50, 12) > 0    # the paper's head width
    # bf16 heads up to 64 wide are padded to 64 (the paper's 50 included); wider ones must keep 16-byte rows
    assert sdp.masked_attn_fwd_workspace_bytes("fm", torch.bfloat16, 4, 2048, 1200, 24, 50, 12) > \
        sdp.masked_attn_fwd_workspace_bytes("fm", torch.bfloat16, 4, 2048, 1200, 24, 64, 12)          # padded weight copies
    assert sdp.masked_attn_fwd_workspace_bytes("fm", torch.bfloat16, 4, 2048, 1536, 24, 84, 12) == 0
    assert L.sdp_masked_attn_saved_head_width(BF16, 50) == 64 and L.sdp_masked_attn_saved_head_width(BF16, 64) == 64
    assert L.sdp_masked_attn_saved_head_width(BF16, 96) == 96 and L.sdp_masked_attn_saved_head_width(F32, 50) == 50
    assert L.sdp_masked_attn_saved_head_width(BF16, 0) == 0 and L.sdp_masked_attn_saved_head_width(9, 64) == 0
    assert sdp.masked_attn_fwd_workspace_bytes("fm", torch.bfloat16, 4, 2048, 1536, 24, 136, 12) == 0  # wider than 128
    assert sdp.masked_attn_bwd_workspace_bytes("fm", torch.bfloat16, 4, 2048, 1532, 24, 64, 12) == 0  # d % 8
    fwd = lambda *a: L.sdp_masked_attn_fwd(*a)
    # mode, dtype, Bt, S, d, H, hd, ph, then X, Wqkv, WoT, head_idx, Y, QKV, O, LSE, ws, ws_bytes, stream
    args = [FM, BF16, 2, 128, 128, 4, 64, 2, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, big, None]
    unsupported, invalid, shape, workspace = -5, -1, -2, -3
    assert fwd(*([2] + args[1:])) == invalid                   # unknown regime
    assert fwd(*(args[:1] + [7] + args[2:])) == invalid        # unknown dtype
    assert fwd(*(args[:6] + [136] + args[7:])) == unsupported  # head width beyond 128
    assert fwd(*(args[:6] + [84] + args[7:])) == shape         # bf16 heads wider than 64: rows must be 16-byte multiples
    assert fwd(*(args[:7] + [5] + args[8:])) == shape          # more held heads than heads
    assert fwd(*(args[:2] + [0] + args[3:])) == invalid        # no sequence
    assert fwd(*(args[:8] + [None] + args[9:])) == invalid     # X missing
    assert fwd(*(args[:11] + [None] + args[12:])) == invalid   # forward masking needs the head list
    assert fwd(*(args[:8] + [ctypes.c_void_p(0x1004)] + args[9:])) == invalid  # misaligned
    assert fwd(*(args[:17] + [ctypes.c_size_t(16), None])) == workspace
    bargs = [FM, BF16, 2, 128, 128, 4, 64, 2] + [FAKE] * 11 + [0, FAKE, big, None]
    assert L.sdp_masked_attn_bwd(*(bargs[:19] + [7] + bargs[20:])) == invalid   # unknown gradient layout
    assert L.sdp_masked_attn_bwd(*(bargs[:20] + [None, big, None])) == workspace
    assert L.sdp_masked_attn_bwd(*(bargs[:6] + [136] + bargs[7:])) == unsupported
    assert L.sdp_masked_attn_bwd(*([BM] + bargs[1:12] + [None] + bargs[13:])) == invalid  # the held heads are needed


def test_block_argument_errors():
    L = sdp.lib()
    f = FAKE
    big = ctypes.c_size_t(1 << 40)
    args_f = [f] * 14
    assert L.sdp_block_fwd(0, 2, 1, 1, 64, 64, 2, 32, 64, *args_f, big, None) == -1          # m not 0 / 1
    assert L.sdp_block_fwd(3, 1, 1, 1, 64, 64, 2, 32, 64, *args_f, big, None) == -1          # unknown mode
    assert L.sdp_block_fwd(0, 1, 1, 1, 64, 60, 2, 32, 64, *args_f, big, None) == -2          # d not a multiple of 8
    assert L.sdp_block_fwd(0, 1, 1, 1, 64, 64, 2, 136, 64, *args_f, big, None) == -5         # head width beyond 128
    assert L.sdp_block_fwd(0, 1, 1, 1, 64, 64, 2, 32, 64, *args_f, ctypes.c_size_t(0), None) == -1  # X, Y, Hm alias
    g = ctypes.c_void_p(0x2000); h = ctypes.c_void_p(0x3000)
    ok = [f, f, f, f, f, f, g, h, f, f, f, f, f, f]
    assert L.sdp_block_fwd(0, 1, 1, 1, 64, 64, 2, 32, 64, *ok, ctypes.c_size_t(0), None) == -3      # workspace too small
    assert L.sdp_block_bwd(1, 0, 7, 1, 1, 64, 64, 2, 32, 64, *([f] * 20), big, None) == -1   # unknown dx_rule
