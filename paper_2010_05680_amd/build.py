"""Compile the HIP sources for gfx950 into paper_2010_05680_amd/libturbo_reduce.so.

Run as `python -m paper_2010_05680_amd.build`.  hipcc cross-compiles without a GPU.
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libturbo_reduce.so")

SOURCES = ["api.hip", "softmax_f32.hip", "softmax_f16.hip", "layernorm_f32.hip", "layernorm_f16.hip", "elementwise.hip", "packed.hip",
           "serving_host.cpp"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-FP32 VALU forms stay off on this part
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    # one remark block per kernel (registers, scratch, occupancy); parsed below, so a kernel that spills fails the build
    "-Rpass-analysis=kernel-resource-usage",
]
RESOURCE_FILE = "kernel_resources.txt"


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _kernel_resources(stderr: str):
    """[(kernel, {field: value})] from hipcc's kernel-resource-usage remarks."""
    kernels = []
    for line in stderr.splitlines():
        m = re.search(r"remark:\s+(.*?) \[-Rpass-analysis=kernel-resource-usage\]", line)
        if not m:
            continue
        key, _, value = m.group(1).partition(":")
        key, value = key.strip(), value.strip()
        if key == "Function Name":
            kernels.append((value, {}))
        elif kernels:
            kernels[-1][1][key] = value
    return kernels


def _compile(src: str, extra=(), obj_dir: str = OBJ_DIR):
    obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *HIPCC_FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{res.stdout}\n{res.stderr}")
    return obj, _kernel_resources(res.stderr)


def build_library(verbose: bool = True, extra_flags=(), lib_path: str = LIB_PATH, obj_dir: str = OBJ_DIR,
                  check_spills: bool = True) -> str:
    """Compile every HIP source and link the shared library.  Always recompiles.

    extra_flags / lib_path / obj_dir build a variant (e.g. -DTURBO_NT_LOADS=0) beside the default library."""
    os.makedirs(obj_dir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        compiled = list(pool.map(lambda s: _compile(s, tuple(extra_flags), obj_dir), SOURCES))
    objs = [obj for obj, _ in compiled]
    kernels = [k for _, ks in compiled for k in ks]
    with open(os.path.join(obj_dir, RESOURCE_FILE), "w") as fh:
        for name, f in kernels:
            fh.write(f"{name} vgpr={f.get('VGPRs')} sgpr={f.get('TotalSGPRs')} scratch={f.get('ScratchSize [bytes/lane]')} "
                     f"sgpr_spill={f.get('SGPRs Spill')} vgpr_spill={f.get('VGPRs Spill')} "
                     f"occupancy={f.get('Occupancy [waves/SIMD]')} lds={f.get('LDS Size [bytes/block]')}\n")
    # every kernel keeps its rows in registers: scratch memory would mean spills, i.e. hidden extra memory traffic
    # (scalar registers parked in vector lanes cost no memory traffic and are not counted)
    spilled = [name for name, f in kernels if f.get("ScratchSize [bytes/lane]", "0") != "0" or
               f.get("VGPRs Spill", "0") != "0"]
    if spilled and check_spills:
        raise RuntimeError("kernels that spill registers:\n  " + "\n  ".join(spilled))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib_path, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stdout}\n{res.stderr}")
    if verbose:
        print(f"built {lib_path}", file=sys.stderr)
    return lib_path


if __name__ == "__main__":
    build_library()
