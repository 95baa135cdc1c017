"""Builds libann.so (HIP kernels for gfx950 + the C-ABI host code) in-tree with hipcc."""
from __future__ import annotations

import concurrent.futures
import glob
import json
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libann.so")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-command-line-argument",
         "-Rpass-analysis=kernel-resource-usage",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-I", INCLUDE, "-I", CSRC]


EXTRA = []  # further hipcc flags for this build (command line: python -m paper_2512_02278_amd.build -DNAME=VALUE ...)
# the routing kernels read every matrix result with the vector ALU: keep the accumulators in VGPRs
PER_FILE = {"route_mfma_u8.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"], "route_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


RESOURCES = {}  # kernel name -> {"VGPRs": .., "ScratchSize": .., "Occupancy": ..}, filled by _compile


def _resources(stderr: str) -> str:
    """Collects the compiler's per-kernel resource remarks; returns what is left of stderr."""
    rest, name = [], None
    for line in stderr.splitlines():
        if "kernel-resource-usage" in line:
            m = re.search(r"remark:\s+(.*?)\s+\[-Rpass", line)
            if m:
                key, _, val = m.group(1).partition(":")
                if key.strip() == "Function Name":
                    name = val.strip()
                    RESOURCES[name] = {}
                elif name:
                    RESOURCES[name][key.strip().split(" [")[0]] = val.strip()
            continue
        if re.match(r"^\s*\d+ \| |^\s*\| |^In file included from|^\s+\d+ remarks? generated", line) or "packed-fp32-ops" in line:
            continue  # source echo of the remarks; hipcc's host pass not knowing the packed-fp32 feature is harmless
        rest.append(line)
    return "\n".join(rest)


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    r = subprocess.run(["hipcc", *FLAGS, *EXTRA, *PER_FILE.get(os.path.basename(src), []), "-c", src, "-o", obj],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr}")
    err = _resources(r.stderr)
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(jobs: int = 8, extra_flags=()) -> str:
    EXTRA[:] = list(extra_flags)
    os.makedirs(OBJ, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, srcs))
    # a search kernel that keeps its list or query in scratch memory runs at half speed: refuse it
    spilled = {k: v for k, v in RESOURCES.items()
               if v.get("ScratchSize", "0") != "0" or v.get("VGPRs Spill", "0") != "0"}
    if spilled:
        raise RuntimeError("kernels using scratch memory: " + ", ".join(f"{k} {v}" for k, v in spilled.items()))
    with open(os.path.join(OBJ, "resources.json"), "w") as f:
        json.dump(RESOURCES, f, indent=1, sort_keys=True)
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


CLANG = "/opt/rocm/llvm/bin/clang"
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
             "-fno-sanitize-recover=undefined"]


def build_host_sanitized() -> str:
    """libann_san.so: the host code (ann_host.hip) under ASan + UBSan, linked with the kernel objects of the
    last build().  For the host-only ABI checks; device code cannot be sanitised on this machine pool."""
    objs = [o for o in sorted(glob.glob(os.path.join(OBJ, "*.hip.o"))) if not o.endswith("ann_host.hip.o")]
    if not objs:
        build()
        objs = [o for o in sorted(glob.glob(os.path.join(OBJ, "*.hip.o"))) if not o.endswith("ann_host.hip.o")]
    host = os.path.join(OBJ, "ann_host.san.o")
    flags = [f for f in FLAGS if f != "-O3" and not f.startswith("-Rpass")]
    r = subprocess.run(["hipcc", *flags, "-O1", "-g", *SAN_FLAGS, "-c", os.path.join(CSRC, "ann_host.hip"), "-o", host],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc (sanitized host pass) failed:\n{r.stderr}")
    lib = os.path.join(OBJ, "libann_san.so")
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                    "-fno-gpu-sanitize", "-o", lib, host, *objs], check=True)
    return lib


if __name__ == "__main__":
    if "--sanitize-host" in sys.argv[1:]:
        print(build_host_sanitized())
    else:
        print(build(extra_flags=sys.argv[1:]))
