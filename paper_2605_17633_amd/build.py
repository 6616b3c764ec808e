"""Builds ``libssam.so`` (the gfx950 HIP library) in-tree with hipcc.

hipcc cross-compiles for gfx950 without a GPU.  Objects go to ``_build/`` (not
committed); the shared library lands beside this file so that it travels with
the source tree.
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libssam.so")
SOURCES = ["tables.hip", "movers.hip", "gemm.hip", "attention.hip", "block.hip", "ends.hip", "probe.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-I" + os.path.join(ROOT, "include"),
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function",
         "-Wno-inline-asm"]     # the window attention kernel names m0 in an asm clobber list (LDS-destination loads)


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    raise RuntimeError("hipcc not found")


_REMARK = re.compile(r"remark:\s+(Function Name|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|Occupancy \[waves/SIMD\]|"
                     r"VGPRs Spill|LDS Size \[bytes/block\]): (\S+)")


def _resources(stderr: str):
    """Per-kernel register, scratch and occupancy figures from the compiler's resource-usage remarks."""
    kernels, cur = [], None
    for line in stderr.splitlines():
        m = _REMARK.search(line)
        if not m:
            continue
        key, val = m.group(1), m.group(2)
        if key == "Function Name":
            cur = {"name": val}
            kernels.append(cur)
        elif cur is not None:
            cur[key.split(" [")[0]] = int(val)
    return kernels


def _compile(src: str, obj: str):
    cmd = [_hipcc(), *FLAGS, "-Rpass-analysis=kernel-resource-usage", "-c", os.path.join(CSRC, src), "-o", obj]
    p = subprocess.run(cmd, capture_output=True, text=True)
    keep, held, in_remark = [], [], False
    for l in p.stderr.splitlines():      # drop the remarks, the source lines quoted under them and their include trails
        if "-Rpass-analysis=kernel-resource-usage" in l:
            held, in_remark = [], True
        elif in_remark and re.match(r"^\s*\d*\s*\|", l):
            pass
        elif l.startswith("In file included from"):
            held.append(l)
            in_remark = False
        elif "is not a recognized feature for this target" in l:
            in_remark = False
        else:
            keep += held + [l]
            held, in_remark = [], False
    err = "\n".join(keep)
    if p.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return _resources(p.stderr)


def build_library(force: bool = True, jobs: int = 6) -> str:
    """Compile every HIP source and link libssam.so.  Returns its path."""
    bdir = os.path.join(ROOT, "_build")
    os.makedirs(bdir, exist_ok=True)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(ROOT, "include", "ssam.h")]
    newest = max(os.path.getmtime(d) for d in deps)
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= newest:
        return LIB
    objs = [os.path.join(bdir, s.replace(".hip", ".o")) for s in SOURCES]
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        per_source = list(ex.map(_compile, SOURCES, objs))
    # The GEMM and attention kernels are written to a register budget (two waves per SIMD): a variant that spills
    # runs at a fraction of its speed and would otherwise go unnoticed.  The figures are kept beside the objects.
    spilled = []
    with open(os.path.join(bdir, "kernel_resources.txt"), "w") as f:
        for src, kernels in zip(SOURCES, per_source):
            for k in kernels:
                f.write(f"{src} {k['name']} vgprs={k.get('VGPRs', -1)} agprs={k.get('AGPRs', -1)} "
                        f"scratch={k.get('ScratchSize', -1)} spill={k.get('VGPRs Spill', -1)} "
                        f"occupancy={k.get('Occupancy', -1)} lds={k.get('LDS Size', -1)}\n")
                if k.get("VGPRs Spill", 0) > 0 and ("gemm_bf16_nt_" in k["name"] or "attn_" in k["name"]):
                    spilled.append(f"{k['name']}: {k['VGPRs Spill']} VGPRs spilled")
    if spilled:
        raise RuntimeError("hot kernels spill registers:\n" + "\n".join(spilled))
    p = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if p.returncode != 0:
        raise RuntimeError("link failed:\n" + p.stderr)
    return LIB


if __name__ == "__main__":
    print(build_library(force=True))
