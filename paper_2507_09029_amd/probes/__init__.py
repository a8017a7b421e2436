"""Stand-alone microbenchmarks behind the hardware figures quoted in the design notes (not part of the library).

    python -m paper_2507_09029_amd.probes            # build them next to their sources (hipcc, gfx950)
    paper_2507_09029_amd/probes/lds_read_rate        # then run on the GPU
    paper_2507_09029_amd/probes/direct_load_rate
"""
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def build_probes():
    built = []
    for src in sorted(glob.glob(os.path.join(HERE, "*.hip"))):
        exe = src[:-4]
        r = subprocess.run([HIPCC, *FLAGS, src, "-o", exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}")
        built.append(exe)
    return built
