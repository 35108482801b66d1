"""Builds libknapattn.so in-tree with hipcc for gfx950.

    python paper_2508_06001_amd/build.py

The shared library is written next to this file.  Nothing is built at import
time: the binding loads what this step produced and fails loudly otherwise.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libknapattn.so")

HIP_SOURCES = ["knap_attn_fwd.hip", "knap_attn_bwd.hip", "knap_ulysses.hip", "knap_api.hip"]
C_SOURCES = ["knap_host.c"]

HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the work-queue tickets are drawn by one lane and first looked at an item later; the atomic
    # optimizer would rewrite the draw into a wave reduction that needs its result at once
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    "-Wno-unused-command-line-argument",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = False, extra_flags=(), out_path: str = LIB_PATH, obj_subdir: str = "_build") -> str:
    hipcc = _hipcc()
    obj_dir = os.path.join(HERE, obj_subdir)
    os.makedirs(obj_dir, exist_ok=True)
    inc = ["-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
    objs = []
    procs = []
    for src in HIP_SOURCES:
        obj = os.path.join(obj_dir, src + ".o")
        cmd = [hipcc] + HIP_FLAGS + list(extra_flags) + inc + ["-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src in C_SOURCES:
        obj = os.path.join(obj_dir, src + ".o")
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-Wall", "-Wextra"] + inc + ["-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("build failed: %s\n%s" % (" ".join(cmd), out))
        if verbose and out.strip():
            print(out)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out_path] + objs + ["-lm"]
    r = subprocess.run(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed: %s\n%s" % (" ".join(link), r.stdout))
    return out_path


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
