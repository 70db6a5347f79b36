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


# The hot kernels issue some MFMAs as inline asm so that their result lands in vector registers.  The compiler
# takes such a result to be there at once; it neither waits before it reads the registers nor keeps them free once
# the value is dead.  The kernels are written so that both hold anyway; this check reads the generated code and
# refuses the build when, on some path, anything touches the result of such an MFMA too soon after it: fewer
# than two further MFMAs and fewer than kMinCycles issue cycles of other instructions in between.
MFMA_ASM_CHECKED = {"attn_fwd.hip", "attn_bwd.hip"}
kMinCycles = 64


def _regs(tok: str) -> set:
    m = re.match(r"([va])\[(\d+):(\d+)\]", tok)
    if m:
        return {(m.group(1), i) for i in range(int(m.group(2)), int(m.group(3)) + 1)}
    m = re.match(r"([va])(\d+)$", tok)
    return {(m.group(1), int(m.group(2)))} if m else set()


def early_touches_of_asm_mfma_results(asm_text: str) -> list:
    """[(kernel, mfma line, touching line, cycles, mfmas between)] for every violation found in `asm_text`."""
    marked = []
    in_asm = False
    for raw in asm_text.splitlines():
        if ";;#ASMSTART" in raw:
            in_asm = True
        elif ";;#ASMEND" in raw:
            in_asm = False
        if in_asm and raw.split(";")[0].strip().startswith("v_mfma"):
            raw = raw.replace("v_mfma", "asm.v_mfma", 1)      # hand-written, as opposed to the compiler's own
        marked.append(raw)
    found = []
    for kernel, lines, labels in _split_kernels("\n".join(marked)):
        found += _scan_kernel(kernel, lines, labels)
    return found


def _scan_kernel(kernel: str, lines: list, labels: dict) -> list:
    out = []
    for i, l in enumerate(lines):
        if not l.startswith("asm.v_mfma"):
            continue                                   # the compiler looks after its own MFMAs
        ops = [t.strip() for t in l.split(None, 1)[1].split(",")]
        dst = _regs(ops[0])
        stack, seen = [(i + 1, 0, 0)], set()
        while stack:
            pos, cycles, mfmas = stack.pop()
            while pos < len(lines) and (cycles < kMinCycles and mfmas < 2):
                if (pos, mfmas) in seen:
                    break
                seen.add((pos, mfmas))
                n = lines[pos]
                name, _, rest = n.partition(" ")
                toks = [t.strip() for t in rest.split(",")] if rest else []
                if name.startswith(("v_mfma", "asm.v_mfma")):
                    if _regs(toks[0]) == dst and _regs(toks[-1]) == dst:
                        break                          # the chain goes on in place: hardware interlocks that
                    if any(_regs(t) & dst for t in toks):
                        out.append((kernel, l, n, cycles, mfmas))
                        break
                    mfmas += 1
                elif name == "s_nop":
                    cycles += int(toks[0]) + 1
                elif name in ("s_branch",):
                    pos = labels.get(toks[0], len(lines))
                    continue
                elif name.startswith("s_cbranch"):
                    if toks[0] in labels:
                        stack.append((labels[toks[0]], cycles + 4, mfmas))
                    cycles += 4
                elif name == "s_endpgm":
                    break
                else:
                    if any(_regs(t) & dst for t in toks):
                        out.append((kernel, l, n, cycles, mfmas))
                        break
                    cycles += 4
                pos += 1
    return out


# The same kernels issue LDS reads as inline asm and wait for them later.  Until that wait the compiler takes the
# destination registers to hold their data already: if it copies or reuses one of them in between (it does when
# it is short of registers, and at control-flow joins) the copy holds stale data.  This check follows every path
# through the generated code of the attention kernels, keeps the LDS operations no s_waitcnt has covered yet,
# and refuses the build if any instruction touches the destination of a read among them.
def _split_kernels(asm_text: str):
    kernel, lines, labels = None, [], {}
    for raw in asm_text.splitlines():
        l = raw.split(";")[0].strip()
        if not l:
            continue
        m = re.match(r"(\S+):$", l)
        if m:
            if not m.group(1).startswith(".L"):
                if kernel is not None:
                    yield kernel, lines, labels
                kernel, lines, labels = m.group(1), [], {}
            else:
                labels[m.group(1)] = len(lines)
            continue
        if kernel is None or l.startswith("."):
            continue
        lines.append(l)
    if kernel is not None:
        yield kernel, lines, labels


def touches_of_lds_reads_in_flight(asm_text: str) -> list:
    """[(kernel, read, touching instruction)] for every violation found in kernels whose name contains `attn_`."""
    out = []
    for kernel, lines, labels in _split_kernels(asm_text):
        if "attn_" not in kernel:
            continue
        found, seen, stack = set(), set(), [(0, ())]
        while stack:
            pos, state = stack.pop()
            fifo = list(state)                         # (position of the LDS operation, registers it writes)
            while pos < len(lines):
                key = (pos, tuple(p for p, _ in fifo))
                if key in seen:
                    break
                seen.add(key)
                l = lines[pos]
                name, _, rest = l.partition(" ")
                toks = [t.strip() for t in rest.split(",")] if rest else []
                if name == "s_waitcnt":
                    m = re.search(r"lgkmcnt\((\d+)\)", l)
                    if m:
                        fifo = fifo[max(0, len(fifo) - int(m.group(1))):]
                elif name.startswith("ds_read"):
                    fifo.append((pos, frozenset(_regs(toks[0]))))
                elif name.startswith(("ds_", "s_load")):
                    fifo.append((pos, frozenset()))    # other LDS operations and scalar loads use the same counter
                elif name == "s_branch":
                    pos = labels.get(toks[0], len(lines))
                    continue
                elif name.startswith("s_cbranch"):
                    if toks[0] in labels:
                        stack.append((labels[toks[0]], tuple(fifo)))
                elif name == "s_endpgm":
                    break
                else:
                    touched = set().union(*[_regs(t) for t in toks]) if toks else set()
                    found |= {(lines[p], l) for p, d in fifo if touched & d}
                pos += 1
        out += [(kernel, a, b) for a, b in sorted(found)]
    return out


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
    asm_procs = []
    for src, stem, extra in UNITS:
        if src in MFMA_ASM_CHECKED:
            asm = os.path.join(CSRC, stem + ".s")
            cmd = [HIPCC, *FLAGS, *extra, "--cuda-device-only", "-S", os.path.join(CSRC, src), "-o", asm]
            asm_procs.append((stem, asm, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for stem, asm, p in asm_procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            sys.stderr.write(out)
            raise RuntimeError(f"hipcc -S failed on {stem}")
        with open(asm) as f:
            text = f.read()
        os.remove(asm)
        stale = touches_of_lds_reads_in_flight(text)
        if stale:
            for k, a, b in stale[:10]:
                sys.stderr.write(f"{stem}: {k}: `{b}` while `{a}` is in flight\n")
            raise RuntimeError(f"{stem}: registers of LDS reads in flight are touched ({len(stale)} places)")
        bad = early_touches_of_asm_mfma_results(text)
        if bad:
            for k, a, b, cyc, nm in bad[:10]:
                sys.stderr.write(f"{stem}: {k}: `{b}` {cyc} cycles and {nm} MFMAs after `{a}`\n")
            raise RuntimeError(f"{stem}: results of hand-written MFMAs are touched too early ({len(bad)} places)")
        if verbose:
            print(f"{stem}: hand-written MFMA results are left alone long enough", flush=True)
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
