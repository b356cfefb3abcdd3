"""Builds libchunkflow.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libchunkflow.so")
SOURCES = ["chunkflow.hip", "simulate.hip", "gemm.hip", "attention.hip", "elementwise.hip", "checksum_noalloc.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-pthread",
         # packed-fp32 VALU forms are kept out of every kernel
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Rpass-analysis=kernel-resource-usage"]


def _resource_usage(lines):
    """Parse hipcc's kernel-resource-usage remarks: {kernel: {field: int}}."""
    usage, cur = {}, None
    for l in lines:
        if "kernel-resource-usage" not in l or "remark:" not in l:
            continue
        body = l.split("remark:", 1)[1].replace("[-Rpass-analysis=kernel-resource-usage]", "").strip()
        if body.startswith("Function Name:"):
            cur = body.split(":", 1)[1].strip()
            usage[cur] = {}
        elif cur is not None and ":" in body:
            k, v = body.rsplit(":", 1)
            try:
                usage[cur][k.strip()] = int(v)
            except ValueError:
                pass
    return usage


def build_library(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    build_dir = os.path.join(HERE, "_build")
    os.makedirs(build_dir, exist_ok=True)
    procs = []
    for src in SOURCES:
        obj = os.path.join(build_dir, src.replace(".hip", ".o"))
        cmd = [hipcc] + [f for f in FLAGS if f != "-shared"] + ["-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        lines = out.splitlines()
        usage = _resource_usage(lines)
        out = "\n".join(l for l in lines if "warning:" in l or "error:" in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n" + "\n".join(lines))
        for kname, u in usage.items():
            # a kernel that touches scratch memory has lost its register arrays: treat as a build error
            if u.get("ScratchSize [bytes/lane]", 0) or u.get("VGPRs Spill", 0):
                raise RuntimeError(f"{src}: kernel {kname} uses scratch memory: {u}")
        if verbose and out.strip():
            print(out, file=sys.stderr)
    link = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-pthread", "-o", LIB] + objs
    r = subprocess.run(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}")
    return LIB


if __name__ == "__main__":
    print(build_library())
