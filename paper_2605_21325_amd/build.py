"""Build libtriinv.so (hand-written HIP for gfx950) in-tree with hipcc.

One translation unit per (C, operand type) pair plus the C-ABI file, compiled in parallel and
linked into paper_2605_21325_amd/libtriinv.so.  Packed-fp32 code generation is switched off
for every device compile.
"""
from __future__ import annotations

import json
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libtriinv.so")
RESOURCES = os.path.join(HERE, "kernel_resources.json")  # registers / scratch / LDS of every kernel, from the compiler

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wno-pass-failed", "-Wno-unused-command-line-argument",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # keep MFMA results in ordinary VGPRs: the kernels post-process every accumulator with vector
         # ALU code, and the accumulator-register form costs one copy instruction per register
         "-mllvm", "-amdgpu-mfma-vgpr-form=1",
         "-Rpass-analysis=kernel-resource-usage"]

# slowest units first so the pool stays busy
UNITS = [
    (f"inst_nb{nb}_op{op}_fwd", "inst.hip", [f"-DTRIINV_INST_NB={nb}", f"-DTRIINV_INST_OP={op}", "-DTRIINV_INST_FWD=1"])
    for nb in (8, 4, 2, 1) for op in (0, 1, 2)
] + [
    (f"inst_nb{nb}_op{op}", "inst.hip", [f"-DTRIINV_INST_NB={nb}", f"-DTRIINV_INST_OP={op}"])
    for nb in (8, 4, 2, 1) for op in (0, 1, 2)
] + [
    (f"solve_nb{nb}_op{op}", "solve.hip", [f"-DTRIINV_INST_NB={nb}", f"-DTRIINV_INST_OP={op}"])
    for nb in (8, 4, 2, 1) for op in (0, 1, 2)
] + [("api", "api.hip", [])]


def _sources_mtime() -> float:
    return max(os.path.getmtime(os.path.join(CSRC, f)) for f in os.listdir(CSRC))


_REMARK = re.compile(r"remark:\s+(Function Name|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|Occupancy \[waves/SIMD\]|"
                     r"VGPRs Spill|LDS Size \[bytes/block\]): (\S+)")


def _parse_resources(stderr: str) -> dict:
    out, cur = {}, None
    for key, val in _REMARK.findall(stderr):
        if key == "Function Name":
            cur = out.setdefault(val, {})
        elif cur is not None:
            cur[{"VGPRs": "vgpr", "AGPRs": "agpr", "ScratchSize [bytes/lane]": "scratch", "Occupancy [waves/SIMD]": "occupancy",
                 "VGPRs Spill": "vgpr_spill", "LDS Size [bytes/block]": "lds"}[key]] = int(val)
    return out


def _compile(unit):
    name, src, defs = unit
    out = os.path.join(OBJ, name + ".o")
    cmd = [HIPCC, *FLAGS, *defs, "-c", os.path.join(CSRC, src), "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {name}:\n{r.stderr[-4000:]}")
    return out, _parse_resources(r.stderr)


def build(force: bool = False, jobs: int = 0) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= _sources_mtime():
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or min(len(UNITS), os.cpu_count() or 4, 16)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        results = list(ex.map(_compile, UNITS))
    objs = [o for o, _ in results]
    resources = {}
    for _, res in results:
        resources.update(res)
    with open(RESOURCES, "w") as f:
        json.dump(dict(sorted(resources.items())), f, indent=0)
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr[-4000:]}")
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
