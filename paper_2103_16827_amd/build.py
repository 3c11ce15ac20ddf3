"""Builds libqasr.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import glob
import os
import re
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


def partial_write_hazards(asm_text: str):
    """Instruction pairs in device assembly where a vector instruction reads a register that the
    instruction just before it wrote through a byte/word selector (`..._sdwa` with `dst_sel` other
    than DWORD).  gfx950 needs one instruction in between; the compiler inserts it for its own
    code but cannot see inside `asm` statements."""
    ins = []
    for l in asm_text.splitlines():
        l = l.strip()
        if not l or l[0] in ";./" or l.endswith(":"):
            continue
        ins.append(l)
    bad = []
    for a, b in zip(ins, ins[1:]):
        if "_sdwa" in a.split()[0] and "dst_sel:" in a and "dst_sel:DWORD" not in a:
            dst = a.split()[1].rstrip(",")
            if b.startswith("v_") and re.search(r"\b" + re.escape(dst) + r"\b", b):
                bad.append((a, b))
    return bad


def source_with_local_includes(src: str, seen=None) -> str:
    """Text of a source file followed by that of every header of this directory it includes."""
    seen = set() if seen is None else seen
    if src in seen or not os.path.exists(src):
        return ""
    seen.add(src)
    with open(src) as f:
        text = f.read()
    for inc in re.findall(r'#include\s+"([^"]+)"', text):
        text += source_with_local_includes(os.path.join(os.path.dirname(src), inc), seen)
    return text


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    procs = []
    sdwa_sources = []
    for src in sources():
        obj = os.path.join(bdir, os.path.basename(src) + ".o")
        cmd = [hipcc, "-x", "hip", "-c", src, "-o", obj] + [f for f in HIPCC_FLAGS if f != "-shared"]
        if "_sdwa" in source_with_local_includes(src):   # hand-written partial register writes: device assembly too
            asm = os.path.join(bdir, os.path.basename(src) + ".gfx950.s")
            acmd = [hipcc, "-x", "hip", "--cuda-device-only", "-S", src, "-o", asm] + \
                   [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC", "-Rpass-analysis=kernel-resource-usage")]
            sdwa_sources.append((src, asm, subprocess.Popen(acmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
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
    for src, asm, pr in sdwa_sources:
        out, _ = pr.communicate()
        if pr.returncode != 0:
            raise RuntimeError(f"no device assembly for {src}:\n{out}")
        with open(asm) as f:
            bad = partial_write_hazards(f.read())
        if bad:
            if os.path.exists(LIB):
                os.remove(LIB)
            raise RuntimeError(f"{asm}: register read right after a partial write: {bad[0][0]} | {bad[0][1]}")
    if not recs:       # no figures parsed (the remark's format changed?): nothing was checked
        if os.path.exists(LIB):
            os.remove(LIB)
        raise RuntimeError("the compiler reported no per-kernel resource usage: the scratch-memory check cannot run")
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
