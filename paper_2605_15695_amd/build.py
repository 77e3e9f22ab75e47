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


if __name__ == "__main__":
    build(verbose=True)
