"""Builds libfcs.so (HIP, gfx950 only) in-tree next to the sources."""
from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfcs.so")
SOURCES = ["fcs_api.hip", "fcs_sim.hip"]

# What the launch geometry relies on: registers per lane at most (four wavefronts per SIMD need 128 for the
# kernel of the FLOW and GREEDY cells), and no scratch memory (state that leaves the registers would put
# memory round trips on a path's instruction chain).
RESOURCE_LIMITS = {"fcs_sim_kernel": {"VGPRs": 128, "ScratchSize [bytes/lane]": 0},
                   "fcs_sim_skip_kernel": {"VGPRs": 128, "ScratchSize [bytes/lane]": 0},
                   "fcs_sim_all_kernel": {"VGPRs": 256, "ScratchSize [bytes/lane]": 0},
                   "fcs_sim_mck_kernel": {"VGPRs": 256, "ScratchSize [bytes/lane]": 0}}


def kernel_resources(remarks: str) -> dict:
    """{kernel: {field: value}} from the compiler's kernel-resource-usage remarks."""
    out, cur = {}, None
    for ln in remarks.splitlines():
        m = re.search(r"remark: Function Name: (\S+)", ln)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z \[\]/]+): (\S+)", ln)
        if m and cur is not None:
            cur[m.group(1).strip()] = m.group(2)
    return out


def build_library(verbose: bool = False, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Rpass-analysis=kernel-resource-usage",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *extra_flags,
           "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stderr)
        raise subprocess.CalledProcessError(r.returncode, cmd)
    res = kernel_resources(r.stderr)
    for kernel, limits in RESOURCE_LIMITS.items():
        found = [v for k, v in res.items() if kernel + "E" in k]   # mangled name: <len><name>E...
        if not found:
            raise RuntimeError(f"no resource remark for {kernel}")
        use = found[0]
        if verbose:
            print(kernel, {k: use.get(k) for k in ("VGPRs", "TotalSGPRs", "ScratchSize [bytes/lane]",
                                                   "Occupancy [waves/SIMD]", "SGPRs Spill")})
        for field, limit in limits.items():
            if int(use[field]) > limit:
                raise RuntimeError(f"{kernel}: {field} = {use[field]} exceeds {limit}")
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
