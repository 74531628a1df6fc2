"""Builds libadapmoe.so (HIP, gfx950) in-tree with hipcc.

The compiler's per-kernel resource remarks are parsed: a kernel that uses scratch memory (register
spills, or a local array indexed with a run-time value) fails the build, because a private segment
has to be set up at every dispatch and costs the decode kernels several microseconds per launch.
The figures of every kernel are written next to the library (kernel_resources.txt)."""
from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libadapmoe.so")
RESOURCES = os.path.join(HERE, "kernel_resources.txt")
SOURCES = ["adapmoe_host.hip", "kernels_gate.hip", "kernels_ffn.hip", "kernels_int4.hip", "kernels_batched.hip", "kernels_misc.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Rpass-analysis=kernel-resource-usage",
         "-Wall", "-Wno-unused-command-line-argument", "-Wno-unused-value"]

_REMARK = re.compile(r"remark:\s+(Function Name|TotalSGPRs|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|Occupancy \[waves/SIMD\]|"
                     r"LDS Size \[bytes/block\]):\s+(\S+)")


def kernel_resources(compiler_output: str) -> dict:
    """{kernel symbol: {field: value}} from the compiler's kernel-resource-usage remarks."""
    res, cur = {}, None
    for line in compiler_output.splitlines():
        m = _REMARK.search(line)
        if not m:
            continue
        key, val = m.group(1), m.group(2)
        if key == "Function Name":
            cur = res.setdefault(val, {})
        elif cur is not None:
            cur[key.split(" [")[0]] = int(val)
    return res


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    resources = {}
    for src, p in procs:
        out, _ = p.communicate()
        resources.update(kernel_resources(out))
        lines, skip = [], 0
        for l in out.splitlines():   # drop the remarks (and the two source lines quoted after each) and the feature warning
            if "kernel-resource-usage" in l:
                skip = 2
            elif skip and re.match(r"\s+(\d+\s+)?\|", l):
                skip -= 1
            elif "packed-fp32-ops" not in l:
                lines.append(l)
        out = "\n".join(lines)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out, file=sys.stderr)
    with open(RESOURCES, "w") as f:
        f.write("kernel | SGPRs | VGPRs | AGPRs | scratch bytes/lane | waves/SIMD | static LDS bytes\n")
        for name in sorted(resources):
            r = resources[name]
            f.write(" | ".join([name] + [str(r.get(k, "?")) for k in
                                         ("TotalSGPRs", "VGPRs", "AGPRs", "ScratchSize", "Occupancy", "LDS Size")]) + "\n")
    if not resources:
        raise RuntimeError("no kernel resource remarks in the compiler output")
    spilled = sorted(n for n, r in resources.items() if r.get("ScratchSize", 0) != 0)
    if spilled:
        raise RuntimeError("kernels using scratch memory (see the module docstring): " + ", ".join(spilled))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    return LIB


if __name__ == "__main__":
    print(build())
