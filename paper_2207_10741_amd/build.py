"""Build libfocused_conv.so in-tree with hipcc for gfx950.

    python -m paper_2207_10741_amd.build
"""
from __future__ import annotations

import concurrent.futures
import glob
import os
import shutil
import subprocess
import sys
import tempfile

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
OUT = os.path.join(_HERE, "libfocused_conv.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # let the compiler not form packed-fp32 instructions on its own
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]

# fc_conv_mfma.hip holds most of the kernel instances; it is compiled as this many units
# (-DFC_MFMA_PART=p), side by side with the other sources
MFMA_SOURCE = "fc_conv_mfma.hip"
MFMA_PARTS = 6


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the packed-fp32 feature name and says so: harmless
    noise = ("packed-fp32-ops", "target feature")
    log = "\n".join(ln for ln in res.stdout.splitlines() if not any(n in ln for n in noise))
    if verbose and log.strip():
        print(log, flush=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed (%d): %s\n%s" % (res.returncode, " ".join(cmd), res.stdout))


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    srcs = sorted(glob.glob(os.path.join(_HERE, "csrc", "*.hip")))
    inc = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(_HERE, "csrc")]
    jobs = max(1, min(int(os.environ.get("MAX_JOBS", "8")), os.cpu_count() or 1, 8))
    tmp = tempfile.mkdtemp(prefix="fc_build_")
    try:
        units = []      # (object file, compile command); the large units first
        for src in srcs:
            name = os.path.basename(src)
            if name == MFMA_SOURCE:
                for part in range(MFMA_PARTS):
                    obj = os.path.join(tmp, "%s.%d.o" % (name, part))
                    units.insert(0, (obj, [hipcc, *HIPCC_FLAGS, *inc, "-DFC_MFMA_PART=%d" % part, "-c", src, "-o", obj]))
            else:
                obj = os.path.join(tmp, name + ".o")
                units.append((obj, [hipcc, *HIPCC_FLAGS, *inc, "-c", src, "-o", obj]))
        with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
            for f in [pool.submit(_run, cmd, verbose) for _, cmd in units]:
                f.result()
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *[o for o, _ in units], "-o", OUT + ".tmp"], verbose)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    os.replace(OUT + ".tmp", OUT)
    return OUT


if __name__ == "__main__":
    build()
    sys.exit(0)
