"""Build libsig.so (the C-ABI library) from csrc/ with hipcc for gfx950.

Run as `python -m paper_2501_08455_amd.build` or through `__graft_entry__.build()`.
Objects go to paper_2501_08455_amd/_build/, the library next to this file.
"""
import json
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsig.so")
RESOURCES = os.path.join(OBJ, "kernel_resources.json")

SOURCES = ["sig_api.hip", "sig_streaming.hip", "sig_onchip_table.hip", "sig_onchip_table_depth2.hip",
           "sig_onchip_table_depth3.hip", "sig_onchip_table_depth4.hip", "sig_onchip_table_depth56.hip", "sig_onchip_table_odd.hip",
           "sig_backward.hip", "sig_backward_segments.hip", "sig_backward_general.hip", "sig_levelscan.hip", "sig_levelscan_rows.hip", "sig_probe.hip"]

# packed FP32 instructions are switched off for every device translation unit
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wno-unused-command-line-argument",
               "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


_RESOURCE = re.compile(r"remark:\s+(Function Name|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|VGPRs Spill|SGPRs Spill|"
                       r"Occupancy \[waves/SIMD\]|LDS Size \[bytes/block\]): (\S+)")


def _compile(src):
    """Compile one translation unit; returns (object path, {kernel: resource usage as the compiler reports it})."""
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc()] + HIPCC_FLAGS + ["-Rpass-analysis=kernel-resource-usage", "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, res.stdout, res.stderr))
    kernels, cur = {}, None
    for key, val in _RESOURCE.findall(res.stderr):
        if key == "Function Name":
            cur = kernels.setdefault(val, {})
        elif cur is not None:
            cur[key.split(" [")[0]] = int(val)
    return obj, kernels


def build(verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        done = list(pool.map(_compile, SOURCES))
    objs = [obj for obj, _ in done]
    # registers, LDS and private memory of every kernel, for the host test that no kernel spills
    with open(RESOURCES, "w") as f:
        json.dump({src: kernels for src, (_, kernels) in zip(SOURCES, done)}, f, indent=0, sort_keys=True)
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (res.stdout, res.stderr))
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
