"""Builds the HIP library for gfx950 in-tree: csrc/*.hip -> libgnn_mi355x.so.

hipcc cross-compiles without a GPU.  Objects go to ``_build/`` (ignored by git),
the shared library next to this file, where ``binding.py`` looks for it.
"""
from __future__ import annotations

import concurrent.futures
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgnn_mi355x.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # keep MFMA accumulators in ordinary VGPRs: with the AGPR form the compiler copied all
    # 64 accumulator registers in and out around every k-tile of the persistent GEMM loop
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    # per-kernel register / scratch / LDS figures as remarks: _compile turns scratch use into an error
    "-Rpass-analysis=kernel-resource-usage",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    cmd = [HIPCC, *FLAGS, "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr}")
    # A kernel whose local arrays end up in scratch (private) memory runs several times slower than
    # the same kernel with them in registers, silently: refuse to build one.
    kernel, offenders, plain = None, [], []
    for line in r.stderr.splitlines():
        if "kernel-resource-usage" in line:
            if "Function Name:" in line:
                kernel = line.split("Function Name:")[1].split("[")[0].strip()
            elif "ScratchSize [bytes/lane]:" in line:
                size = int(line.split("ScratchSize [bytes/lane]:")[1].split("[")[0])
                if size > 0:
                    offenders.append(f"{kernel}: {size} bytes per lane")
        elif "packed-fp32-ops" not in line and line.strip():
            plain.append(line)
    # the remark lines are followed by source excerpts ("  13 | ...", "     | ^"): drop those too
    plain = [l for l in plain if not l.lstrip().startswith("|") and not (l.strip()[:1].isdigit() and " | " in l)]
    if offenders:
        raise RuntimeError(f"{os.path.basename(src)}: kernels with scratch memory:\n  " + "\n  ".join(offenders))
    if plain:
        sys.stderr.write("\n".join(plain) + "\n")
    return obj


def build(verbose: bool = True, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, srcs))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.check_call(cmd)
    if verbose:
        print(f"built {LIB} from {len(srcs)} sources")
    return LIB


if __name__ == "__main__":
    build()
