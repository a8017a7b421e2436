"""Workload and summariser for rocprofv3 counter runs (HBM traffic, MFMA utilisation).

Run under the profiler, it launches, in this order and a few times each: a plain device-to-device copy of a
known size (the calibration kernel: it reads and writes exactly `copy_bytes`) and the kernels under study
at their benchmark size.  FETCH_SIZE / WRITE_SIZE of the kernels under study are scaled by
(known bytes / counted bytes) of the copy.

    python3 paper_2507_09029_amd/traffic_probe.py avg                       # coverage average, 1B-parameter workload
    python3 paper_2507_09029_amd/traffic_probe.py mlp [workload] [zeros]    # one worker's fwd+bwd (default: the
                                                                            # bench's headline workload); `zeros`
                                                                            # runs it on all-zero X, dY and weights
    python3 paper_2507_09029_amd/traffic_probe.py summarize FETCH.csv WRITE.csv SHAPES.json WORKLOAD
        # reads the two counter_collection.csv files of rocprofv3 --pmc FETCH_SIZE / --pmc WRITE_SIZE runs of the
        # commands above and the launch shapes the probe wrote, prints a table and updates
        # profiles/hbm_traffic_recorded.json (the figures bench.py reports as roofline.traffic)
    python3 paper_2507_09029_amd/traffic_probe.py counters FILE.csv [FILE.csv ...]
        # per-kernel means of every counter in rocprofv3 counter_collection.csv files
"""
import csv
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_recorded.json")
COPY_NAME = "__amd_rocclr_copyBuffer"

# call-site name of each contraction <-> the <epilogue, op> template arguments of its kernel symbol
SITE_OF = {(2, 0): "mlp_gate_up", (0, 1): "mlp_down", (3, 2): "mlp_dact", (1, 3): "mlp_dx", (0, 4): "mlp_dw",
           (0, 6): "mlp_dw"}  # op 6: the weight-gradient launch with the tiles of its last round cut in depth


def kernel_site(kernel_name):
    """'mlp_dw' etc. for an sdp_gemm_kernel<BM, BN, WM, WN, EPI, OP> symbol, 'coverage_grad_avg' for the storing
    average, the calibration copy's own name, else None."""
    if COPY_NAME in kernel_name:
        return COPY_NAME
    if "avg_rows_kernel<1, 0>" in kernel_name or "avg_rows_kernel<true, 0>" in kernel_name:
        return "coverage_grad_avg"
    if "tail_reduce_kernel" in kernel_name:
        return "mlp_dw_reduce"
    if "sdp_gemm_kernel<" in kernel_name:
        args = kernel_name.split("sdp_gemm_kernel<", 1)[1].split(">", 1)[0].split(",")
        try:
            return SITE_OF.get((int(args[4]), int(args[5])))
        except (IndexError, ValueError):
            return None
    return None


def read_counters(paths):
    """{site: {counter: [values per dispatch]}} from counter_collection.csv files; the pseudo-counter
    "duration_ns" holds End_Timestamp - Start_Timestamp of each dispatch (once per dispatch)."""
    out = {}
    for path in paths:
        seen = set()
        with open(path, newline="") as f:
            for r in csv.DictReader(f):
                site = kernel_site(r["Kernel_Name"])
                if not site:
                    continue
                out.setdefault(site, {}).setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
                key = (path, r["Dispatch_Id"])
                if key not in seen:
                    seen.add(key)
                    out[site].setdefault("duration_ns", []).append(float(r["End_Timestamp"]) - float(r["Start_Timestamp"]))
    return out


def mean(v):
    return sum(v) / len(v)


def summarize(fetch_csv, write_csv, shapes_json, workload):
    fetch, write = read_counters([fetch_csv]), read_counters([write_csv])
    with open(shapes_json) as f:
        shapes = json.load(f)
    copy_kib = shapes["copy_bytes"] / 1024.0

    def calibration(v):
        # torch issues smaller copies through the same kernel; the 1 GiB ones are the largest by far
        big = [x for x in v if x > 0.9 * max(v)]
        return mean(big)

    f_scale = copy_kib / calibration(fetch[COPY_NAME]["FETCH_SIZE"])
    w_scale = copy_kib / calibration(write[COPY_NAME]["WRITE_SIZE"])
    print(f"calibration: FETCH_SIZE x {f_scale:.3f}, WRITE_SIZE x {w_scale:.3f} (1 GiB copy)")
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        rec = {}
    rec.setdefault(workload, {})
    print("| kernel | launch | FETCH KiB | WRITE KiB | read MB | written MB | total MB |")
    print("|---|---|---|---|---|---|---|")
    for site in fetch:
        if site == COPY_NAME or site not in write:
            continue
        fk, wk = mean(fetch[site]["FETCH_SIZE"]), mean(write[site]["WRITE_SIZE"])
        fb, wb = fk * 1024 * f_scale, wk * 1024 * w_scale
        launch = shapes["launch"].get(site)
        rec[workload][site] = {"fetch_bytes": round(fb), "write_bytes": round(wb), "launch": launch}
        print(f"| {site} | {launch} | {fk:,.0f} | {wk:,.0f} | {fb / 1e6:.1f} | {wb / 1e6:.1f} | {(fb + wb) / 1e6:.1f} |")
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(rec, f, indent=1, sort_keys=True)
        f.write("\n")


def counters(paths):
    data = read_counters(paths)
    for site, cs in data.items():
        n = len(next(iter(cs.values())))
        print(f"{site}: {n} dispatches")
        for c in sorted(cs):
            print(f"    {c:34s} {mean(cs[c]):18.0f}")


def run(what, workload_name, zeros):
    import torch

    import paper_2507_09029_amd as sdp
    import workloads

    reps = 3
    copy_bytes = 1 << 30
    src = torch.empty(copy_bytes, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    for _ in range(reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(f"calibration copy: {copy_bytes} bytes read, {copy_bytes} bytes written per launch", flush=True)
    shapes = {"copy_bytes": copy_bytes, "launch": {}}
    if what == "avg":
        c = workloads.CONFIG5
        name = c.name
        mask = sdp.sample_masks_host(c.K, c.R, c.p, c.mask_seed, False).cuda()
        grads = workloads.grad_buffers(c.K, c.R, c.D, c.sigma, "bf16", device="cuda")
        out = torch.empty((c.R, c.D), dtype=torch.float32, device="cuda")
        cov = torch.empty((c.R,), dtype=torch.uint8, device="cuda")
        for _ in range(reps):
            sdp.coverage_grad_avg(grads, mask, out=out, cov=cov)
        torch.cuda.synchronize()
        shapes["launch"]["coverage_grad_avg"] = None
        print(f"{c.name}: algorithmic bytes per launch {c.algorithmic_bytes} "
              f"(read {c.K * c.p * c.D * 2 + c.K * c.R}, write {c.R * c.D * 4 + c.R})", flush=True)
    else:
        w = workloads.MLP_CONFIGS[workload_name]
        name = w.name + ("_zeros" if zeros else "")
        Wd = [t.cuda() for t in workloads.mlp_weights(w)]
        X, dY = (t.cuda() for t in workloads.mlp_batch(w, 0))
        if zeros:
            for t in Wd + [X, dY]:
                t.zero_()
        mask, idx, pos, cov = sdp.make_masks(w.K, w.F, w.p, w.mask_seed, True)
        sdp.profile_enable(True)  # only so that the library remembers the launch shapes
        for _ in range(reps):
            Y, G, U = sdp.masked_mlp_fwd(w.mode, X, *Wd, idx[0])
            sdp.masked_mlp_bwd(w.mode, X, dY, *Wd, idx[0], G, U)
        torch.cuda.synchronize()
        for site in set(SITE_OF.values()):
            shapes["launch"][site] = sdp.profile_launch_shape(site)
        sdp.profile_enable(False)
        print(f"{name}: one worker fwd+bwd x{reps}", flush=True)
    os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
    with open(os.path.join(ROOT, "gpurun_out", f"traffic_shapes_{name}.json"), "w") as f:
        json.dump(shapes, f)


def main():
    what = sys.argv[1] if len(sys.argv) > 1 else "avg"
    if what == "summarize":
        return summarize(*sys.argv[2:6])
    if what == "counters":
        return counters(sys.argv[2:])
    import bench

    rest = sys.argv[2:]
    zeros = "zeros" in rest
    names = [r for r in rest if r != "zeros"]
    run(what, names[0] if names else bench.DEFAULT_WORKLOAD, zeros)


if __name__ == "__main__":
    main()
