"""Workload for HBM-traffic counter runs (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE).

Launches, in this order and a few times each: a plain device-to-device copy of a known size (the
calibration kernel: it must read and write exactly `copy_bytes` each) and the kernel under study at
its benchmark size.  The counters of the kernel under study are scaled by (known bytes / counted
bytes) of the copy.

    python -m paper_2507_09029_amd.traffic_probe avg        # coverage average, 1B-parameter workload
    python -m paper_2507_09029_amd.traffic_probe mlp        # one worker's fwd+bwd at the bench workload
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main():
    import torch

    import paper_2507_09029_amd as sdp
    import workloads

    what = sys.argv[1] if len(sys.argv) > 1 else "avg"
    reps = 3
    copy_bytes = 1 << 30
    src = torch.empty(copy_bytes, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    for _ in range(reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(f"calibration copy: {copy_bytes} bytes read, {copy_bytes} bytes written per launch", flush=True)
    if what == "avg":
        c = workloads.CONFIG5
        mask = sdp.sample_masks_host(c.K, c.R, c.p, c.mask_seed, False).cuda()
        grads = workloads.grad_buffers(c.K, c.R, c.D, c.sigma, "bf16", device="cuda")
        out = torch.empty((c.R, c.D), dtype=torch.float32, device="cuda")
        cov = torch.empty((c.R,), dtype=torch.uint8, device="cuda")
        for _ in range(reps):
            sdp.coverage_grad_avg(grads, mask, out=out, cov=cov)
        torch.cuda.synchronize()
        print(f"{c.name}: algorithmic bytes per launch {c.algorithmic_bytes} "
              f"(read {c.K * c.p * c.D * 2 + c.K * c.R}, write {c.R * c.D * 4 + c.R})", flush=True)
    else:
        w = workloads.CONFIG2
        Wd = [t.cuda() for t in workloads.mlp_weights(w)]
        X, dY = (t.cuda() for t in workloads.mlp_batch(w, 0))
        mask, idx, pos, cov = sdp.make_masks(w.K, w.F, w.p, w.mask_seed, True)
        for _ in range(reps):
            Y, G, U = sdp.masked_mlp_fwd(w.mode, X, *Wd, idx[0])
            sdp.masked_mlp_bwd(w.mode, X, dY, *Wd, idx[0], G, U)
        torch.cuda.synchronize()
        print(f"{w.name}: one worker fwd+bwd x{reps}", flush=True)


if __name__ == "__main__":
    main()
