"""Builds libqasr.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libqasr.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
    # packed-fp32 instruction forms are kept off on this platform
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # matrix-core results stay in ordinary vector registers (no copies through the accumulator file)
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    "-Wall", "-Wno-unused-command-line-argument",
    # per-kernel register / scratch / LDS figures as compiler remarks: kept in resource_usage.txt
    "-Rpass-analysis=kernel-resource-usage",
]
RESOURCES = os.path.join(HERE, "resource_usage.txt")


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip"))) + sorted(glob.glob(os.path.join(CSRC, "*.cpp")))


def kernels_using_scratch(recs):
    """Names of the kernels whose resource record (name, then `Key:value` strings as the compiler
    printed them, blanks removed) does not say `ScratchSize[bytes/lane]:0`."""
    return [r[0] for r in recs if "ScratchSize[bytes/lane]:0" not in r[1:]]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    procs = []
    for src in sources():
        obj = os.path.join(bdir, os.path.basename(src) + ".o")
        cmd = [hipcc, "-x", "hip", "-c", src, "-o", obj] + [f for f in HIPCC_FLAGS if f != "-shared"]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    remarks = []
    for src, pr in procs:
        out, _ = pr.communicate()
        remarks += [l for l in out.splitlines() if "[-Rpass-analysis=kernel-resource-usage]" in l]
        kept, skip = [], 0
        for l in out.splitlines():
            if "kernel-resource-usage" in l:
                skip = 2                       # the remark's echo of the source line and its caret
            elif skip and (l.lstrip().startswith("|") or "|" in l[:8]):
                skip -= 1
            elif "packed-fp32-ops" not in l and l.strip():
                kept.append(l)
        out = "\n".join(kept)
        if pr.returncode != 0:
            failed = True
            print(f"--- {src} failed:\n{out}", file=sys.stderr)
        elif out and verbose:
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    # one line per kernel: name, then the figures the compiler reported for it
    recs, cur = [], None
    for l in remarks:
        body = l.split("remark:", 1)[1].replace("[-Rpass-analysis=kernel-resource-usage]", "").strip()
        if body.startswith("Function Name:"):
            cur = [body[len("Function Name:"):].strip()]
            recs.append(cur)
        elif cur is not None and ":" in body:
            cur.append(body.replace(" ", ""))
    with open(RESOURCES, "w") as f:
        for r in recs:
            f.write(" ".join(r) + "\n")
    # The pipelined kernels count their own vector-memory requests; a spill adds requests nobody
    # counted and moves registers that loads in flight still own.  Such a build must never run.
    spilled = kernels_using_scratch(recs)
    if spilled:
        if os.path.exists(LIB):
            os.remove(LIB)
        raise RuntimeError("kernels use scratch memory (register spills): " + ", ".join(spilled))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
