"""Build libquamba.so (HIP, gfx950) in-tree: `python -m paper_2410_13229_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libquamba.so")
SOURCES = ["api.hip", "gemm_i8.hip", "elementwise.hip", "scan.hip", "hadamard.hip", "calibrate.hip", "model.hip", "decode_fused.hip", "gemm_xfmt.hip", "microbench.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + os.path.join(ROOT, "include"),
         "-I" + CSRC, "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Rpass-analysis=kernel-resource-usage"]
# Kernels that count their own outstanding loads (explicit vmcnt waits) must not spill: scratch
# accesses share that counter and would make the waits release too early.
NO_SPILL = ("gemm_i8_dma_kernel",)


def _check_spills(stderr: str) -> None:
    """Read the compiler's per-kernel resource remarks; refuse spills in the NO_SPILL kernels."""
    name = None
    for line in stderr.splitlines():
        if "remark: Function Name:" in line:
            name = line.split("Function Name:")[1].split()[0]
        elif name and ("ScratchSize [bytes/lane]:" in line or "VGPRs Spill:" in line or "SGPRs Spill:" in line):
            val = int(line.split(":")[-1].split()[0])
            if val != 0 and any(k in name for k in NO_SPILL):
                raise RuntimeError("kernel %s spills (%s): its explicit vmcnt waits would be wrong"
                                   % (name, line.split("remark:")[1].strip()))


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s\n%s" % (" ".join(cmd), r.stdout, r.stderr))
    _check_spills(r.stderr)
    keep, skip = [], 0
    for l in r.stderr.splitlines():  # drop the resource remarks and the harmless feature warning
        if "is not a recognized feature" in l:
            continue
        if "kernel-resource-usage" in l:
            skip = 2  # the remark is followed by a source line and a caret line
            continue
        if skip:
            skip -= 1
            continue
        keep.append(l)
    return "\n".join(keep)


def build(verbose: bool = False) -> str:
    """Compile every .hip source for gfx950 and link libquamba.so next to this file."""
    os.makedirs(OBJ, exist_ok=True)
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]

    def one(pair):
        src, obj = pair
        return _run([HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])

    with ThreadPoolExecutor(max_workers=min(10, len(SOURCES))) as ex:
        for msg in ex.map(one, zip(SOURCES, objs)):
            if verbose and msg.strip():
                print(msg, file=sys.stderr)
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
