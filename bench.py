#!/usr/bin/env python3
"""Benchmark of the SDP masked-MLP hot path on one MI355X.

A step is one pass of the whole path over one batch of seeded synthetic input, everything resident
in HBM: mask -> index compaction, then for each of the K simulated workers (run back to back on one
stream) the masked SwiGLU MLP forward and backward writing its weight gradients into that worker's
full-size bf16 gradient buffer, then the coverage-normalised average of the K buffers.

Prints ONE JSON line.  The headline workload is the largest one-GPU configuration, the 1B-LLaMA-like
MLP under backward masking (dense forward and dX, weight gradients on each worker's mask); `value` is
its active TFLOP/s (12 T d F + 6 T d p per worker and step there, 18 T d p under forward masking; the
dense work the method avoids is not counted).  `roofline` is for the kernel that takes most of the
step; `other_configs` holds the same measurement for the 500M-like and the 1B-like forward-masking
workloads; `grad_avg` reports the HBM-bound average alone at 1B-parameter scale; `attention` reports
one worker's head-masked attention block (not part of `value`); `cpu_baseline` is the fp64 oracle
timed on this host on a bounded sample of the headline workload, `cpu_baselines_other` the same for
the average and for the small fp32 configuration (one thread and all threads).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA peak (published: 2.5 PFLOP/s)
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E peak (published: 8 TB/s)
PEAK_FP32_VECTOR_TFLOPS = 157.3  # 256 CUs x 128 fp32 FMA lanes x 2 flop x 2.4 GHz

# HBM-side bytes per launch come from rocprofv3 counter runs (FETCH_SIZE, then WRITE_SIZE, each scaled by what
# the same counter reads for a 1 GiB copy).  Counters cannot be read from inside this process: the file below is
# written by `python -m paper_2507_09029_amd.traffic_probe summarize ...` from those runs and records, next to each
# figure, the tile shape and tile order the kernel was launched with.  A figure is reported only while the
# kernel still launches that way; otherwise `traffic` is null.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_recorded.json")
DEFAULT_WORKLOAD = "config4_bf16_bm_1B"


def recorded_traffic(workload, kernel, shape):
    """Recorded L2 <-> fabric bytes per launch of `kernel` at `workload`, or None when there is no record or
    the launch configuration (`shape`, from sdp_profile_launch_shape; None for kernels that have none) differs."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec_all = json.load(f).get(workload, {})
    except (OSError, ValueError):
        return None
    rec = rec_all.get(kernel)
    if not rec:
        return None
    if rec.get("launch") != shape:
        return None
    total = rec["fetch_bytes"] + rec["write_bytes"]
    if kernel + "_reduce" in rec_all:  # the kernel that adds the partial tiles of a launch cut in depth
        total += rec_all[kernel + "_reduce"]["fetch_bytes"] + rec_all[kernel + "_reduce"]["write_bytes"]
    return total


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the sub-objects for the other bf16 MLP workloads (default line only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-grad-avg-1b", action="store_true", help="skip the 1B-parameter average measurement")
    ap.add_argument("--avg-steps", type=int, default=20)
    ap.add_argument("--no-attention", action="store_true", help="skip the head-masked attention block measurement")
    ap.add_argument("--attention-only", action="store_true",
                    help="measure the head-masked attention block alone and print its object (for profiler runs)")
    ap.add_argument("--events", type=int, default=1, help="1: per-kernel HIP events recorded during the timed steps")
    ap.add_argument("--graph", type=int, default=0, help="1: capture one step into a HIP graph and replay it (no per-kernel events)")
    ap.add_argument("--streams", type=int, default=1,
                    help="HIP streams the K simulated workers are spread over (worker k on stream k %% S)")
    return ap.parse_args()


def flops_per_launch(name, w):
    n = w.p if w.mode == "fm" else w.F
    return {
        "mlp_gate_up": 4 * w.T * w.d * n,
        "mlp_down": 2 * w.T * w.d * n,
        "mlp_dact": 2 * w.T * w.d * n,
        "mlp_dx": 4 * w.T * w.d * n,
        "mlp_dw": 6 * w.T * w.d * w.p,  # one batched launch for dW1, dW3, dW2T
    }.get(name)


def _omp_threads(n=None):
    """Thread count the oracle's OpenMP loops use; n sets it (the oracle library links the same libgomp)."""
    import ctypes

    gomp = ctypes.CDLL("libgomp.so.1")
    if n is not None:
        gomp.omp_set_num_threads(int(n))
    return int(gomp.omp_get_max_threads())


def cpu_baseline(w, target_flop=6e11):
    """The oracle as it stands, timed on this host on a bounded token slice of worker 0's batch (cost is linear in
    the number of token rows): about target_flop of work, 10-30 s on 16 threads."""
    import oracle
    import workloads

    rows = int(min(w.T, max(256, target_flop / (w.active_flop_per_worker / w.T))))
    rows -= rows % 256 if rows > 256 else 0
    W = [workloads.to_f64(t) for t in workloads.mlp_weights(w)]
    X, dY = workloads.mlp_batch(w, 0, rows=rows)
    mask = oracle.make_masks(w.K, w.F, w.p, w.mask_seed, True)[0]
    X, dY = workloads.to_f64(X), workloads.to_f64(dY)
    cores = _omp_threads()
    t0 = time.perf_counter()
    oracle.worker_step(w.mode, mask, X, dY, *W)
    dt = time.perf_counter() - t0
    flop = w.active_flop_per_worker * rows / w.T
    return {
        "value": flop / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
        "sample": f"{w.name}: worker 0, first {rows} of {w.T} token rows, full d and F, fp64, {dt:.2f} s; "
                  f"active flops counted as for the GPU",
    }


def cpu_baselines_other():
    """The oracle beside the other workloads: the coverage average of the 1B-parameter workload on a row slice
    (cost is linear in the rows), and the whole small fp32 configuration on one thread and on all threads."""
    import numpy as np

    import oracle
    import workloads

    out = {}
    cores = _omp_threads()
    c = workloads.CONFIG5
    rows = 16384
    mask = np.ascontiguousarray(oracle.make_masks(c.K, c.R, c.p, c.mask_seed, False)[:, :rows])
    g = [workloads.bf16_bits(t) for t in workloads.grad_buffers(c.K, rows, c.D, c.sigma, "bf16")]
    t0 = time.perf_counter()
    oracle.gated_average(g, mask)
    dt = time.perf_counter() - t0
    nbytes = int(mask.sum()) * c.D * 2 + rows * c.D * 4 + c.K * rows + rows
    out["config5_avg_1B"] = {
        "value": nbytes / dt / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
        "sample": f"first {rows} of {c.R} rows of the {c.K} buffers (row length {c.D}), bf16 in, fp64 out, {dt:.2f} s; "
                  f"bytes counted as for the GPU (covered rows read, fp32-sized output written)",
    }
    del g
    w = workloads.CONFIG1
    W = [workloads.to_f64(t) for t in workloads.mlp_weights(w)]
    masks = oracle.make_masks(w.K, w.F, w.p, w.mask_seed, True)
    batches = [tuple(workloads.to_f64(t) for t in workloads.mlp_batch(w, k)) for k in range(w.K)]
    for label, n in (("one_thread", 1), ("all_threads", cores)):
        _omp_threads(n)
        t0 = time.perf_counter()
        for k in range(w.K):
            oracle.worker_step(w.mode, masks[k], *batches[k], *W)
        dt = time.perf_counter() - t0
        out[f"config1_f32_fm_{label}"] = {
            "value": w.K * w.active_flop_per_worker / dt / 1e12, "unit": "TFLOP/s", "cores": n, "kind": "oracle",
            "sample": f"all {w.K} workers' forward + backward at full size, fp64, {dt:.3f} s",
        }
    _omp_threads(cores)
    return out


def bench_grad_avg_1b(sdp, torch, steps):
    import workloads

    c = workloads.CONFIG5
    mask_host = sdp.sample_masks_host(c.K, c.R, c.p, c.mask_seed, False)
    mask = mask_host.cuda()
    grads = workloads.grad_buffers(c.K, c.R, c.D, c.sigma, "bf16", device="cuda")
    out = torch.empty((c.R, c.D), dtype=torch.float32, device="cuda")
    cov = torch.empty((c.R,), dtype=torch.uint8, device="cuda")
    for _ in range(3):
        sdp.coverage_grad_avg(grads, mask, out=out, cov=cov)
    torch.cuda.synchronize()
    sdp.profile_reset()
    sdp.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        sdp.coverage_grad_avg(grads, mask, out=out, cov=cov)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    prof = sdp.profile_read()
    sdp.profile_enable(False)
    calls, ms = prof["coverage_grad_avg"]
    kern = ms / calls * 1e-3
    gbs = c.algorithmic_bytes / kern / 1e9
    res = {
        "workload": c.name, "K": c.K, "rows": c.R, "row_len": c.D, "covered_rows_per_worker": c.p,
        "algorithmic_bytes": c.algorithmic_bytes, "ms_per_call": kern * 1e3, "ms_per_call_wall": wall * 1e3,
        "value": gbs, "unit": "GB/s",
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                     "traffic": recorded_traffic(c.name, "coverage_grad_avg", None)},
    }
    # what plain streaming sustains on this machine (context for the fractions of the 8 TB/s figure; the library's path
    # never runs these kernels): read-only over the first worker's gradient buffer, and a copy of it into `out`
    res["hbm_streaming_ceiling"] = {
        "read_only_gbs": sdp.probe_hbm_gbs(grads[0]), "copy_gbs": sdp.probe_hbm_gbs(grads[0], out),
        "bytes": grads[0].numel() * 2,
        "note": "16-byte non-temporal accesses, 5 launches each; copy = bytes read + bytes written per second",
    }
    # the squared norm of the average alone (what gradient clipping needs before the fused update): reads the
    # covered gradient rows, writes nothing
    sq = torch.empty((1,), dtype=torch.float64, device="cuda")
    for _ in range(2):
        sdp.coverage_grad_sqnorm(grads, mask, out=sq)
    torch.cuda.synchronize()
    sdp.profile_reset()
    sdp.profile_enable(True)
    nsq = max(3, steps // 2)
    for _ in range(nsq):
        sdp.coverage_grad_sqnorm(grads, mask, out=sq)
    torch.cuda.synchronize()
    prof = sdp.profile_read()
    sdp.profile_enable(False)
    calls, ms = prof["coverage_grad_sqnorm"]
    kern_sq = ms / calls * 1e-3
    rbytes = c.K * c.p * c.D * 2 + c.K * c.R
    res["sqnorm"] = {
        "algorithmic_bytes": rbytes, "ms_per_call": kern_sq * 1e3,
        "roofline": {"bound": "hbm", "achieved": rbytes / kern_sq / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": rbytes / kern_sq / 1e9 / PEAK_HBM_GBS, "traffic": None},
        "note": "covered gradient rows (bf16) + masks read, one fp64 number written",
    }
    # the same pass with AdamW fused in: besides the covered gradient rows it reads and writes the fp32
    # parameters and both moments of every covered row once
    del out
    covered = int((mask_host.sum(dim=0) > 0).sum())
    theta = torch.randn((c.R, c.D), device="cuda") * 0.02
    m = torch.zeros((c.R, c.D), device="cuda")
    v = torch.zeros((c.R, c.D), device="cuda")
    hp = dict(lr=4e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    for t in range(1, 3):
        sdp.coverage_avg_adamw(grads, mask, theta, m, v, step=t, cov=cov, **hp)
    torch.cuda.synchronize()
    sdp.profile_reset()
    sdp.profile_enable(True)
    nst = max(3, steps // 2)
    for t in range(3, 3 + nst):
        sdp.coverage_avg_adamw(grads, mask, theta, m, v, step=t, cov=cov, **hp)
    torch.cuda.synchronize()
    prof = sdp.profile_read()
    sdp.profile_enable(False)
    calls, ms = prof["coverage_avg_adamw"]
    kern = ms / calls * 1e-3
    abytes = c.K * c.p * c.D * 2 + c.K * c.R + c.R + 6 * covered * c.D * 4
    res["adamw_fused"] = {
        "algorithmic_bytes": abytes, "covered_rows": covered, "ms_per_call": kern * 1e3,
        "roofline": {"bound": "hbm", "achieved": abytes / kern / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": abytes / kern / 1e9 / PEAK_HBM_GBS, "traffic": None},
        "note": "covered gradient rows (bf16) + masks read; theta, m, v (fp32) of covered rows read and written",
    }
    return res


def bench_attention(sdp, torch, steps, w=None):
    """One worker's head-masked attention block (forward + backward) at the 500M-like width: not part of `value`."""
    import workloads

    w = w or workloads.ATTN_500M
    Wqkv, WoT = (t.cuda() for t in workloads.attn_weights(w))
    mask, idx, pos, cov = sdp.make_masks(w.K, w.H, w.ph, w.mask_seed, True)
    X, dY = (t.cuda() for t in workloads.attn_batch(w, 0))
    wsf = torch.empty(sdp.masked_attn_fwd_workspace_bytes("fm", X.dtype, w.Bt, w.S, w.d, w.H, w.hd, w.ph), dtype=torch.uint8, device="cuda")
    wsb = torch.empty(sdp.masked_attn_bwd_workspace_bytes("fm", X.dtype, w.Bt, w.S, w.d, w.H, w.hd, w.ph), dtype=torch.uint8, device="cuda")
    E = w.ph * w.hd
    Es = w.ph * sdp.attn_saved_head_width(X.dtype, w.hd)  # saved tensors: narrow heads are padded to 64 columns
    fo = (torch.empty((w.T, w.d), dtype=X.dtype, device="cuda"), torch.empty((w.T, 3 * Es), dtype=X.dtype, device="cuda"),
          torch.empty((w.T, Es), dtype=X.dtype, device="cuda"), torch.empty((w.Bt, w.ph, w.S), dtype=torch.float32, device="cuda"))
    bo = (torch.empty((w.T, w.d), dtype=X.dtype, device="cuda"), torch.empty((3, E, w.d), dtype=X.dtype, device="cuda"),
          torch.empty((E, w.d), dtype=X.dtype, device="cuda"))

    def one_pass():
        for k in range(w.K):
            Y, QKV, O, LSE = sdp.masked_attn_fwd("fm", w.Bt, w.S, w.hd, X, Wqkv, WoT, idx[k], out=fo, ws=wsf)
            sdp.masked_attn_bwd("fm", w.Bt, w.S, w.hd, X, dY, Wqkv, WoT, idx[k], QKV, O, LSE, out=bo, ws=wsb)

    for _ in range(2):
        one_pass()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        one_pass()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    sdp.profile_reset()
    sdp.profile_enable(True)
    one_pass()
    torch.cuda.synchronize()
    prof = sdp.profile_read()
    sdp.profile_enable(False)
    kern = {name: tot / calls for name, (calls, tot) in prof.items() if name.startswith("attn_")}
    core_fwd = 2 * w.Bt * w.ph * w.S * w.S * w.hd
    core_bwd = 5 * w.Bt * w.ph * w.S * w.S * w.hd
    core_ms = kern["attn_core_fwd"] + kern["attn_core_bwd_dq"] + kern["attn_core_bwd_dkv"]
    return {
        "workload": w.name, "sequences": w.Bt, "seq_len": w.S, "d_model": w.d, "heads": w.H, "head_dim": w.hd,
        "held_heads": w.ph, "workers_simulated": w.K, "active_flop_per_worker": w.active_flop_per_worker,
        "ms_per_worker": ms / w.K, "value": w.active_flop_per_worker * w.K / (ms * 1e-3) / 1e12, "unit": "TFLOP/s",
        "kernels_avg_ms": kern,
        "core": {"forward_tflops": core_fwd / (kern["attn_core_fwd"] * 1e-3) / 1e12,
                 "backward_tflops": core_bwd / ((core_ms - kern["attn_core_fwd"]) * 1e-3) / 1e12,
                 "roofline": {"bound": "mfma", "achieved": (core_fwd + core_bwd) / (core_ms * 1e-3) / 1e12,
                              "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                              "frac": (core_fwd + core_bwd) / (core_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, "traffic": None},
                 "forward_backward_tflops": (core_fwd + core_bwd) / (core_ms * 1e-3) / 1e12,
                 "note": "causal: the half of the S x S products that is computed is counted (2 S^2 hd per head forward, 5 S^2 hd backward)"},
        "vendor_attention_yardstick": vendor_attention_yardstick(torch, w) if w.hd % 8 == 0 else None,
    }


def vendor_attention_yardstick(torch, w):
    """What torch's own fused causal attention (scaled_dot_product_attention on its flash and memory-efficient
    back ends) reaches on this machine at the core's shape (held heads only), flops counted like the core's: context
    for the core's roofline fraction, not part of the path (the library never calls it)."""
    import torch.nn.functional as F
    from torch.nn.attention import SDPBackend, sdpa_kernel

    gen = torch.Generator(device="cuda")
    gen.manual_seed(11)
    shape = (w.Bt, w.ph, w.S, w.hd)
    q, k, v = (torch.randn(shape, generator=gen, device="cuda").to(torch.bfloat16).requires_grad_(True) for _ in range(3))
    do = torch.randn(shape, generator=gen, device="cuda").to(torch.bfloat16)
    fwd_flop = 2 * w.Bt * w.ph * w.S * w.S * w.hd
    out = {}
    for name, backend in (("flash", SDPBackend.FLASH_ATTENTION), ("mem_efficient", SDPBackend.EFFICIENT_ATTENTION)):
        def run(bwd):
            with sdpa_kernel(backend):
                o = F.scaled_dot_product_attention(q, k, v, is_causal=True)
            if bwd:
                o.backward(do)
                q.grad = k.grad = v.grad = None

        try:
            res = {}
            for bwd in (False, True):
                for _ in range(3):
                    run(bwd)
                torch.cuda.synchronize()
                reps = 10
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    run(bwd)
                e1.record()
                torch.cuda.synchronize()
                res["fwd_bwd_ms" if bwd else "fwd_ms"] = e0.elapsed_time(e1) / reps
            res["forward_tflops"] = fwd_flop / (res["fwd_ms"] * 1e-3) / 1e12
            res["forward_backward_tflops"] = 3.5 * fwd_flop / (res["fwd_bwd_ms"] * 1e-3) / 1e12
            out[name] = res
        except RuntimeError as e:  # a back end this torch build does not have for the shape
            out[name] = {"unavailable": str(e)[:120]}
    out["note"] = ("torch.nn.functional.scaled_dot_product_attention, bf16, causal, [sequences][held heads][S][head_dim]; "
                   "10 back-to-back calls; flops: 2 S^2 hd per head forward, 5 S^2 hd backward (causal half)")
    return out


def vendor_gemm_yardstick(torch, w):
    """What the vendor's bf16 contraction (torch.matmul, i.e. hipBLASLt / rocBLAS) reaches on this machine at the plain
    shapes of this workload's launches, on data with the benchmark's statistics: context for the roofline
    fractions, not part of the path (the library never calls it)."""
    n = w.p if w.mode == "fm" else w.F
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7)
    out = {}
    for name, (M, N, K) in {"gate_up_shape": (w.T, 2 * n, w.d), "down_shape": (w.T, w.d, n), "dw_shape_one_problem": (w.p, w.d, w.T)}.items():
        A = torch.randn((M, K), generator=gen, device="cuda").to(torch.bfloat16)
        B = (torch.randn((N, K), generator=gen, device="cuda") * 0.02).to(torch.bfloat16)
        for _ in range(3):
            C = A @ B.t()
        torch.cuda.synchronize()
        reps = 10
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            C = A @ B.t()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        out[name] = {"M": M, "N": N, "K": K, "ms": ms, "tflops": 2.0 * M * N * K / (ms * 1e-3) / 1e12}
        del A, B, C
    out["note"] = "torch.matmul, bf16 in, fp32 accumulate, A [M][K] x B [N][K]^T, N(0,1) x N(0, 0.02^2) operands; 10 back-to-back calls"
    return out


def bench_block(sdp, torch, steps):
    """One worker's pass through one residual block (attention + MLP) under block-level masking at the 500M-like
    width: the running block (m = 1), the backward-masked block whose gradient still passes through it, and the
    skipped block.  Not part of `value`."""
    import workloads

    a, m = workloads.ATTN_500M, workloads.CONFIG2
    assert a.d == m.d and a.T == m.T
    Wqkv, WoT = (t.cuda() for t in workloads.attn_weights(a))
    W1, W3, W2T = (t.cuda() for t in workloads.mlp_weights(m))
    X, dY = (t.cuda() for t in workloads.attn_batch(a, 0))
    dt = X.dtype
    ws_f = torch.empty(sdp.block_fwd_workspace_bytes(dt, a.Bt, a.S, a.d, a.H, a.hd, m.F), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(sdp.block_bwd_workspace_bytes(dt, a.Bt, a.S, a.d, a.H, a.hd, m.F), dtype=torch.uint8, device="cuda")
    Y, saved = sdp.block_fwd("bm", 1, a.Bt, a.S, a.hd, X, Wqkv, WoT, W1, W3, W2T, ws=ws_f)
    fo = (Y,) + tuple(saved)
    dX, grads = sdp.block_bwd("bm", 1, a.Bt, a.S, a.hd, X, dY, Wqkv, WoT, W1, W3, W2T, saved, ws=ws_b)
    bo = (dX,) + tuple(grads)

    def timed(fn):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    def run(mode, bit, rule):
        skipped_fwd = mode == "fm" and not bit  # nothing is saved then, and only Y is written

        def f():
            _, sv = sdp.block_fwd(mode, bit, a.Bt, a.S, a.hd, X, Wqkv, WoT, W1, W3, W2T, out=Y if skipped_fwd else fo, ws=ws_f)
            sdp.block_bwd(mode, bit, a.Bt, a.S, a.hd, X, dY, Wqkv, WoT, W1, W3, W2T, sv, dx_rule=rule,
                          out=bo if bit else (dX,), ws=ws_b)
        return f

    T, d, F, E = a.T, a.d, m.F, a.H * a.hd
    proj = 2 * T * d * E
    core_f, core_b = 2 * a.Bt * a.H * a.S * a.S * a.hd, 5 * a.Bt * a.H * a.S * a.S * a.hd
    fwd = 4 * proj + core_f + 6 * T * d * F            # q, k, v, out projections; causal core; gate, up, down
    bwd_dx = 4 * proj + core_b + 6 * T * d * F         # dout, dX of the projections, core backward; dact, dX of the MLP
    bwd_dw = 4 * proj + 6 * T * d * F                  # the seven weight gradients
    full = timed(run("bm", 1, "through"))
    through = timed(run("bm", 0, "through"))
    skip_bwd = timed(run("bm", 0, "skip"))
    skipped = timed(run("fm", 0, "through"))
    return {
        "workload": f"block: {a.name} + dense MLP of {m.name}", "tokens": T, "d_model": d, "heads": a.H, "head_dim": a.hd, "d_ff": F,
        "flop": {"forward": fwd, "backward_dx": bwd_dx, "backward_dw": bwd_dw},
        "running_block_m1": {"ms": full, "tflops": (fwd + bwd_dx + bwd_dw) / (full * 1e-3) / 1e12},
        "backward_masked_m0_dx_through": {"ms": through, "tflops": (fwd + bwd_dx) / (through * 1e-3) / 1e12},
        "backward_masked_m0_dx_skip": {"ms": skip_bwd, "tflops": fwd / (skip_bwd * 1e-3) / 1e12},
        "forward_masked_m0_skipped": {"ms": skipped, "note": "two copies of T x d"},
        "unit": "ms per forward + backward of one block on one worker; TFLOP/s of the flops that case runs",
    }


def bench_mlp(sdp, torch, w, a, steps, warmup):
    """One MLP workload: W warm-up steps, an untimed per-kernel survey, then exactly `steps` timed steps."""
    import workloads

    tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    dev = "cuda"

    # ---- resident inputs ----
    Wd = [t.cuda() for t in workloads.mlp_weights(w)]
    gen = torch.Generator(device=dev)
    gen.manual_seed(workloads.BASE_SEED)
    Xs = [torch.randn((w.T, w.d), generator=gen, device=dev, dtype=torch.float32).to(tdt) for _ in range(w.K)]
    dYs = [torch.randn((w.T, w.d), generator=gen, device=dev, dtype=torch.float32).to(tdt) for _ in range(w.K)]
    mask, idx, pos, cov = sdp.make_masks(w.K, w.F, w.p, w.mask_seed, True)
    row_mask = mask.repeat(1, 3).contiguous()
    n = w.p if w.mode == "fm" else w.F
    S = max(1, min(a.streams, w.K))
    main = torch.cuda.current_stream()
    streams = [main] + [torch.cuda.Stream() for _ in range(S - 1)]  # default priority
    per = []
    for _ in range(S):
        per.append(dict(
            Y=torch.empty((w.T, w.d), dtype=tdt, device=dev), G=torch.empty((w.T, n), dtype=tdt, device=dev),
            U=torch.empty((w.T, n), dtype=tdt, device=dev), dX=torch.empty((w.T, w.d), dtype=tdt, device=dev),
            ws_f=torch.empty(sdp.masked_mlp_fwd_workspace_bytes(w.mode, tdt, w.T, w.d, w.F, w.p), dtype=torch.uint8, device=dev),
            ws_b=torch.empty(sdp.masked_mlp_bwd_workspace_bytes(w.mode, tdt, w.T, w.d, w.F, w.p), dtype=torch.uint8, device=dev)))
    bufs = [torch.zeros((3 * w.F, w.d), dtype=tdt, device=dev) for _ in range(w.K)]
    avg = torch.empty((3 * w.F, w.d), dtype=torch.float32, device=dev)
    avg_cov = torch.empty((3 * w.F,), dtype=torch.uint8, device=dev)
    ws_i = torch.empty(max(sdp.index_masks_workspace_bytes(w.K, w.F), 256), dtype=torch.uint8, device=dev)
    idx2 = torch.empty_like(idx)
    pos2 = torch.empty_like(pos)
    cnt2 = torch.empty((w.K,), dtype=torch.int32, device=dev)
    cov2 = torch.empty_like(cov)
    L = sdp.lib()
    ev_idx = torch.cuda.Event()
    ev_done = [torch.cuda.Event() for _ in range(S)]

    def step():
        nonlocal main
        st = L.sdp_index_masks(w.K, w.F, mask.data_ptr(), idx2.data_ptr(), w.p, pos2.data_ptr(), cnt2.data_ptr(),
                               cov2.data_ptr(), ws_i.data_ptr(), ws_i.numel(), main.cuda_stream)
        assert st == 0, st
        if S > 1:
            ev_idx.record(main)
        for k in range(w.K):
            b, q = bufs[k], per[k % S]
            with torch.cuda.stream(streams[k % S]):
                if S > 1 and k < S and k % S != 0:
                    streams[k % S].wait_event(ev_idx)
                sdp.masked_mlp_fwd(w.mode, Xs[k], *Wd, idx2[k], out=(q["Y"], q["G"], q["U"]), ws=q["ws_f"])
                sdp.masked_mlp_bwd(w.mode, Xs[k], dYs[k], *Wd, idx2[k], q["G"], q["U"], dw_layout="scatter",
                                   out=(q["dX"], b[: w.F], b[w.F: 2 * w.F], b[2 * w.F:]), ws=q["ws_b"])
        for i in range(1, S):
            ev_done[i].record(streams[i])
            main.wait_event(ev_done[i])
        sdp.coverage_grad_avg(bufs, row_mask, out=avg, cov=avg_cov)

    run_step = step
    events = a.events
    if a.graph:
        # one eager step first (first-launch set-up is not capturable), then capture and replay
        step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        cap = torch.cuda.Stream()
        with torch.cuda.stream(cap):
            saved_main, saved_streams0 = main, streams[0]
            main = cap
            streams[0] = cap
            with torch.cuda.graph(graph, stream=cap):
                step()
            main, streams[0] = saved_main, saved_streams0
        run_step = graph.replay
        events = 0
    for _ in range(warmup):
        run_step()
    torch.cuda.synchronize()

    # ---- survey (untimed): a few steps with HIP events around EVERY kernel, to find the kernel that
    # takes most of the step and to fill the per-kernel table.  Events between back-to-back kernels
    # cost about a tenth of the step, so the timed region below only brackets that one kernel.
    def per_kernel(prof, nsteps, step_ms):
        out = {}
        for name, (calls, ms) in prof.items():
            f = flops_per_launch(name, w)
            avg_ms = ms / calls
            out[name] = {"launches_per_step": calls / nsteps, "avg_ms": avg_ms, "share_of_step": ms / nsteps / step_ms}
            if f:
                out[name]["tflops"] = f / (avg_ms * 1e-3) / 1e12
                out[name]["launch"] = sdp.profile_launch_shape(name)
        return out

    kernels, dominant = {}, None
    if events and not a.graph:
        nsurvey = max(1, min(3, steps))
        sdp.profile_filter(None)
        sdp.profile_reset()
        sdp.profile_enable(True)
        t0 = time.perf_counter()
        for _ in range(nsurvey):
            run_step()
        torch.cuda.synchronize()
        survey_ms = (time.perf_counter() - t0) / nsurvey * 1e3
        kernels = per_kernel(sdp.profile_read(), nsurvey, survey_ms)
        sdp.profile_enable(False)
        gemm = {k: v for k, v in kernels.items() if "tflops" in v}
        if gemm:
            dominant = max(gemm, key=lambda k: gemm[k]["share_of_step"])

    # ---- timed region: exactly `steps` steps; HIP events (on the launch stream) around the dominant kernel only
    sdp.profile_reset()
    if dominant:
        sdp.profile_filter(dominant)
        sdp.profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = sdp.profile_read() if dominant else {}
    sdp.profile_enable(False)
    sdp.profile_filter(None)

    ms_per_step = elapsed / steps * 1e3
    flop_step = w.K * w.active_flop_per_worker
    value = flop_step / (ms_per_step * 1e-3) / 1e12

    roofline = None
    if dominant and dominant in prof:
        calls, ms = prof[dominant]
        avg_ms = ms / calls
        # a weight-gradient launch whose last round is cut in depth is followed by the kernel that adds the partial
        # tiles: its time (from the survey; it is not timed live) counts against the launch
        reduce_ms = kernels.get(dominant + "_reduce", {}).get("avg_ms", 0.0)
        ach = flops_per_launch(dominant, w) / ((avg_ms + reduce_ms) * 1e-3) / 1e12
        # the fp32 path (config 1, a correctness configuration) runs on the vector ALUs, not on the matrix cores
        bound, peak = ("mfma", PEAK_BF16_TFLOPS) if w.dtype == "bf16" else ("alu", PEAK_FP32_VECTOR_TFLOPS)
        shape = kernels[dominant].get("launch")
        roofline = {"bound": bound, "kernel": dominant, "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                    "frac": ach / peak,
                    "traffic": recorded_traffic(w.name, dominant, shape) if S == 1 else None,
                    "traffic_unit": "bytes per launch (L2 <-> fabric, rocprofv3 FETCH_SIZE + WRITE_SIZE, recorded for this "
                                    "launch configuration in profiles/hbm_traffic_recorded.json; null if none matches)",
                    "launch": shape, "avg_launch_ms": avg_ms, "reduce_kernel_ms": reduce_ms,
                    "launches_timed": calls, "flop_per_launch": flops_per_launch(dominant, w),
                    "share_of_step": ms / steps / ms_per_step}

    # forward and backward separately (sums of the survey's per-kernel means, per worker)
    fwd_names = ("mlp_wt_fwd", "mlp_gate_up", "mlp_down")
    fwd_bwd = None
    if kernels:
        f = sum(v["avg_ms"] * v["launches_per_step"] / w.K for k, v in kernels.items() if k in fwd_names)
        b = sum(v["avg_ms"] * v["launches_per_step"] / w.K for k, v in kernels.items() if k.startswith("mlp_") and k not in fwd_names)
        fwd_bwd = {"forward": f, "backward": b}

    res = {
        "value": value, "unit": "TFLOP/s", "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "dtype": w.dtype,
        "config": {"workload": w.name, "mode": w.mode, "tokens": w.T, "d_model": w.d, "d_ff": w.F, "active_neurons": w.p,
                   "workers_simulated": w.K, "active_flop_per_step": flop_step, "streams": S},
        "frac_of_bf16_peak": value / PEAK_BF16_TFLOPS if w.dtype == "bf16" else None,
        "roofline": roofline,
        "kernels": kernels,
        "fwd_bwd_ms_per_worker": fwd_bwd,
    }
    return res, Xs[0]


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build measures one GPU only (K workers are simulated back to back on it); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2507_09029_amd as sdp
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    L = sdp.lib()
    torch.cuda.set_device(0)
    if a.attention_only:
        print(json.dumps({"attention": bench_attention(sdp, torch, max(2, a.steps // 4)),
                          "attention_paper_width": bench_attention(sdp, torch, max(2, a.steps // 4), workloads.ATTN_500M_HD50),
                          "block": bench_block(sdp, torch, max(2, a.steps // 4))}))
        return
    w = workloads.MLP_CONFIGS[a.workload]
    res, x0 = bench_mlp(sdp, torch, w, a, a.steps, a.warmup)
    rec = {
        "metric": "masked-MLP fwd+bwd active TFLOP/s (% bf16 MFMA peak) + grad-avg GB/s (% HBM)",
        "value": res["value"], "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": res["config"],
        "frac_of_bf16_peak": res["frac_of_bf16_peak"],
        "roofline": res["roofline"],
        "kernels": res["kernels"],
        "fwd_bwd_ms_per_worker": res["fwd_bwd_ms_per_worker"],
        "kernels_note": "per-kernel table from an untimed survey of up to 3 steps with HIP events around every kernel "
                        "(that instrumentation slows a step by about a tenth); roofline is timed live in the K timed steps",
    }
    # practical ceiling of the matrix cores: the same MFMA instruction with no memory traffic, on operands with
    # this workload's statistics (N(0,1) rounded to bf16) and on all-zero operands (the clock the chip holds
    # under MFMA load depends on the operand bits)
    if w.dtype == "bf16":
        nop = L.sdp_probe_mfma_operand_bytes() // 2
        rnd = x0.reshape(-1)[:nop].contiguous()
        rec["mfma_ceiling"] = {
            "random_operands_tflops": sdp.probe_mfma_tflops(rnd),
            "zero_operands_tflops": sdp.probe_mfma_tflops(torch.zeros_like(rnd)),
            "random_operands_tflops_32x32x16": sdp.probe_mfma_tflops(rnd, shape=32),
            "published_peak_tflops": PEAK_BF16_TFLOPS,
            "note": "v_mfma_f32_16x16x32_bf16 loop (the instruction the contractions use; the 32x32x16 form for comparison), "
                    "8 waves per CU, no memory traffic; measured live",
        }
        rec["vendor_gemm_yardstick"] = vendor_gemm_yardstick(torch, w)
    del res, x0
    torch.cuda.empty_cache()
    # the other bf16 MLP workloads, measured the same way (their own steps; not part of `value`)
    if a.workload == DEFAULT_WORKLOAD and not a.no_other_configs:
        rec["other_configs"] = {}
        for name, st in (("config3_bf16_fm_1B", max(3, a.steps // 2)), ("config2_bf16_fm_500M", a.steps)):
            r, _ = bench_mlp(sdp, torch, workloads.MLP_CONFIGS[name], a, st, max(1, min(a.warmup, 3)))
            rec["other_configs"][name] = r
            del r, _
            torch.cuda.empty_cache()
    if not a.no_grad_avg_1b:
        rec["grad_avg"] = bench_grad_avg_1b(sdp, torch, a.avg_steps)
    if not a.no_attention:
        rec["attention"] = bench_attention(sdp, torch, max(2, a.steps // 4))
        rec["attention_paper_width"] = bench_attention(sdp, torch, max(2, a.steps // 4), workloads.ATTN_500M_HD50)
        rec["block"] = bench_block(sdp, torch, max(2, a.steps // 4))
    if not a.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(w)
        rec["cpu_baselines_other"] = cpu_baselines_other()
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
