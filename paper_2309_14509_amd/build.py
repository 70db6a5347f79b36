"""Builds libulysses.so (gfx950) in-tree with hipcc.  No GPU is needed to build."""
from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libulysses.so")
SOURCES = ["api.cpp", "layout.hip", "attn_fwd.hip", "attn_bwd.hip", "attn_d256.hip"]
HEADERS = ["internal.h", "attn_launch.h", "attn_common.h", os.path.join("..", "..", "include", "ulysses.h")]
# (source, object stem, extra flags): the attention sources are compiled once per element type
UNITS = [("api.cpp", "api", []), ("layout.hip", "layout", []),
         ("attn_fwd.hip", "attn_fwd", []), ("attn_bwd.hip", "attn_bwd", []),
         ("attn_d256.hip", "attn_d256", []),
         ("attn_fwd.hip", "attn_fwd_f16", ["-DULY_BUILD_F16=1"]), ("attn_bwd.hip", "attn_bwd_f16", ["-DULY_BUILD_F16=1"]),
         ("attn_d256.hip", "attn_d256_f16", ["-DULY_BUILD_F16=1"])]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
         # packed-fp32 VALU forms are kept off for every device function of this library
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# The attention kernels issue LDS reads by hand (inline asm) and wait for them later.  The compiler does
# not know that such a register is still being written, so a spill or reload of it would save or
# restore stale data: these kernels must compile without any scratch memory.
NO_SCRATCH = {"attn_fwd.hip", "attn_bwd.hip"}
RESOURCE_FLAG = "-Rpass-analysis=kernel-resource-usage"


def scratch_bytes(compiler_output: str) -> dict:
    """{mangled kernel name: scratch bytes per lane} from hipcc's kernel-resource-usage remarks."""
    found, name = {}, None
    for line in compiler_output.splitlines():
        m = re.search(r"remark: Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"remark:\s+ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and name is not None:
            found[name] = int(m.group(1))
    return found


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compile every translation unit and link the shared library.  Returns its path."""
    if not force and not is_stale():
        return LIB
    objs = []
    procs = []
    for src, stem, extra in UNITS:
        obj = os.path.join(CSRC, stem + ".o")
        cmd = [HIPCC, *FLAGS, *extra, *([RESOURCE_FLAG] if src in NO_SCRATCH else []), "-c", os.path.join(CSRC, src),
               "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, stem, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, stem, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            sys.stderr.write(out)
            raise RuntimeError(f"hipcc failed on {src} ({stem})")
        if src in NO_SCRATCH:
            usage = scratch_bytes(out)
            if not usage:
                raise RuntimeError(f"no kernel resource report for {stem}: cannot verify that it uses no scratch")
            bad = {k: v for k, v in usage.items() if v != 0}
            if bad:
                raise RuntimeError(f"{stem}: kernels with hand-issued LDS reads must not use scratch memory: {bad}")
            if verbose:
                print(f"{stem}: {len(usage)} kernels, no scratch memory", flush=True)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
