from . import build_probes

for exe in build_probes():
    print(exe)
