"""Builds libpcsr.so (gfx950) in-tree with hipcc.  `python -m paper_2605_15695_amd.build`."""
from __future__ import annotations

import concurrent.futures
import os
import pathlib
import subprocess

PKG = pathlib.Path(__file__).resolve().parent
CSRC = PKG / "csrc"
OBJ = PKG / "_build"
LIB = PKG / "libpcsr.so"
BASELINE_LIB = PKG / "libpcsr_baseline.so"

HIPCC = "/opt/rocm/bin/hipcc"
COMMON = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-command-line-argument"]
# fp32 atomics as hardware instructions; packed fp32 instructions disabled
DEVICE = ["--offload-arch=gfx950", "-munsafe-fp-atomics",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
SOURCES = ["pcsr_kernels.hip", "pcsr_build_gpu.hip", "pcsr_api.cpp", "pcsr_host.cpp", "pcsr_reorder.cpp"]


def _compile(src: str) -> pathlib.Path:
    obj = OBJ / (src + ".o")
    cmd = [HIPCC, *COMMON]
    if src.endswith(".hip"):
        cmd += DEVICE + os.environ.get("PCSR_EXTRA_HIPCC_FLAGS", "").split()
    cmd += ["-c", str(CSRC / src), "-o", str(obj)]
    r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr}")
    return obj


def build(verbose: bool = False) -> pathlib.Path:
    OBJ.mkdir(exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", *map(str, objs), "-o", str(LIB),
           "-lpthread"]
    subprocess.run(cmd, check=True)
    # vendor baseline used by the benchmarks (links hipSPARSE; not part of libpcsr.so)
    base = _compile("baseline_hipsparse.cpp")
    probe = _compile("probe_gather.hip")
    alg1 = _compile("baseline_alg1.hip")
    subprocess.run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", str(base), str(probe), str(alg1), "-o",
                    str(BASELINE_LIB),
                    "-L/opt/rocm/lib", "-lhipsparse", "-Wl,-rpath,/opt/rocm/lib"], check=True)
    if verbose:
        print(LIB, BASELINE_LIB)
    return LIB


def resources() -> str:
    """Registers, scratch and occupancy of every kernel in pcsr_kernels.hip as the compiler
    reports them (-Rpass-analysis=kernel-resource-usage), as a markdown table."""
    import re

    OBJ.mkdir(exist_ok=True)
    cmd = [HIPCC, *COMMON, *DEVICE, "-Rpass-analysis=kernel-resource-usage", "-c", str(CSRC / "pcsr_kernels.hip"),
           "-o", str(OBJ / "resources.o")]
    r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    if r.returncode != 0:
        raise RuntimeError(r.stderr)
    blocks = re.split(r"remark: Function Name: ", r.stderr)[1:]
    names = subprocess.run(["c++filt"], input="\n".join(b.split()[0] for b in blocks), capture_output=True,
                           text=True).stdout.strip().split("\n")
    rows = []
    for b, name in zip(blocks, names):
        def field(key):
            m = re.search(key + r": (\d+)", b)
            return int(m.group(1)) if m else -1
        short = name.replace("void pcsr::(anonymous namespace)::", "").replace("pcsr::(anonymous namespace)::", "")
        short = short.split("(")[0]
        rows.append((short, field("    VGPRs"), field("TotalSGPRs"), field(r"ScratchSize \[bytes/lane\]"),
                     field(r"Occupancy \[waves/SIMD\]")))
    rows.sort()
    lines = ["| kernel instance | VGPRs | SGPRs | scratch bytes/lane | waves/SIMD the registers allow |",
             "|---|---|---|---|---|"]
    lines += [f"| `{n}` | {v} | {sg} | {sc} | {occ} |" for n, v, sg, sc, occ in rows]
    return "\n".join(lines)


if __name__ == "__main__":
    import sys

    if "--resources" in sys.argv:
        print(resources())
    else:
        build(verbose=True)
