"""Builds libmagicube.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import hashlib
import os
import re
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libmagicube.so")
SOURCES = ["format_host.cpp", "api.hip", "spmm_kernels.hip", "spmm_slab_kernels.hip", "probe_kernels.hip", "sddmm_kernels.hip", "softmax_kernels.hip", "attention_kernels.hip", "attention_pad_kernels.hip", "attention_scores_kernels.hip",
           "quant_kernels.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # per-kernel register / scratch / LDS figures as compiler remarks (parsed below)
    "-Rpass-analysis=kernel-resource-usage",
    # packed fp32 VALU forms are kept out of generated code on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    # the asynchronous-copy helper writes M0 from inline assembly and says so in its clobber list
    "-Wno-inline-asm",
]


def source_id() -> str:
    """Twelve hex digits that change with any source file or compiler flag of the library; mc_version() carries
    them, so that a stored profile can say which build it was taken from."""
    h = hashlib.sha256(" ".join(FLAGS).encode())
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".cpp", ".h")):
            with open(os.path.join(CSRC, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read())
    with open(os.path.join(os.path.dirname(PKG), "include", "magicube.h"), "rb") as f:
        h.update(f.read())
    return h.hexdigest()[:12]


def build_library(verbose: bool = False, jobs: int = 4) -> str:
    """Compiles every source, checks the kernels' resource usage (see check_resources) and links the library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs, objs, table = [], [], []
    sid = source_id()
    for src in SOURCES:
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc, *FLAGS, *([f'-DMC_SOURCE_ID="{sid}"'] if src == "api.hip" else []),
               "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
        if len(procs) >= jobs:
            _wait(procs, verbose, table)
    _wait(procs, verbose, table)
    check_resources(table)
    with open(os.path.join(objdir, "kernel_resources.txt"), "w") as f:
        f.write(format_resources(table))
    with open(os.path.join(objdir, "kernel_resources_summary.txt"), "w") as f:
        f.write(summarize_resources(table))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


_REMARK = re.compile(r"remark:\s+(.*?)\s*\[-Rpass-analysis=kernel-resource-usage\]")


def parse_resources(src: str, compiler_output: str):
    """One dict per kernel of a translation unit from the compiler's resource-usage remarks."""
    kernels, cur = [], None
    for line in compiler_output.splitlines():
        m = _REMARK.search(line)
        if not m:
            continue
        text = m.group(1)
        if text.startswith("Function Name:"):
            cur = {"source": src, "name": text.split(":", 1)[1].strip()}
            kernels.append(cur)
        elif cur is not None and ":" in text:
            key, val = text.rsplit(":", 1)
            cur[key.strip()] = val.strip()
    return kernels


def _demangle(names):
    import shutil
    filt = shutil.which("llvm-cxxfilt") or shutil.which("c++filt")
    if not filt or not names:
        return list(names)
    out = subprocess.run([filt], input="\n".join(names), stdout=subprocess.PIPE, text=True, check=True).stdout
    return [n.replace("(anonymous namespace)::", "").replace("void ", "", 1) for n in out.splitlines()]


def check_resources(table) -> None:
    """Fails the build if a kernel that overlaps hand-counted waits with untracked copies uses scratch.

    Sources that issue asynchronous global -> LDS copies from inline assembly (copy16_to_lds) order them
    with counted s_waitcnt instructions.  That is only sound while the compiler keeps every loaded
    register where the load put it: a spill to scratch between a load and its wait has produced stale
    column indices and an out-of-bounds gather before.  Such kernels must therefore report no scratch
    and no spilled registers."""
    guarded = set()
    for src in SOURCES:
        with open(os.path.join(CSRC, src)) as f:
            text = f.read()
        for inc in re.findall(r'#include "([^"]+)"', text):      # kernels that live in a header of this directory
            if inc != "lds_async.h" and os.path.exists(os.path.join(CSRC, inc)):
                with open(os.path.join(CSRC, inc)) as f:
                    text += f.read()
        if "copy16_to_lds(" in text:
            guarded.add(src)
    bad = [k for k in table if k["source"] in guarded and
           (int(k.get("ScratchSize [bytes/lane]", 0)) or int(k.get("VGPRs Spill", 0)) or int(k.get("SGPRs Spill", 0)))]
    if bad:
        names = _demangle([k["name"] for k in bad])
        raise RuntimeError("kernels with hand-counted waits must not spill: " +
                           "; ".join(f"{n} (scratch {k.get('ScratchSize [bytes/lane]')} B/lane, VGPR spills "
                                     f"{k.get('VGPRs Spill')})" for n, k in zip(names, bad)))


def format_resources(table) -> str:
    names = _demangle([k["name"] for k in table])
    rows = ["source                 VGPRs AGPRs SGPRs scratch spillV LDS_bytes waves/SIMD  kernel"]
    for n, k in sorted(zip(names, table), key=lambda t: (t[1]["source"], t[0])):
        rows.append(f"{k['source']:<22} {k.get('VGPRs', '?'):>5} {k.get('AGPRs', '?'):>5} {k.get('TotalSGPRs', '?'):>5} "
                    f"{k.get('ScratchSize [bytes/lane]', '?'):>7} {k.get('VGPRs Spill', '?'):>6} "
                    f"{k.get('LDS Size [bytes/block]', '?'):>9} {k.get('Occupancy [waves/SIMD]', '?'):>10}  {n}")
    return "\n".join(rows) + "\n"


def summarize_resources(table) -> str:
    """One line per kernel template: number of instantiations and the extremes over them."""
    names = _demangle([k["name"] for k in table])
    fam = {}
    for n, k in zip(names, table):
        key = (k["source"], n.split("<", 1)[0].split("(", 1)[0])
        fam.setdefault(key, []).append(k)
    rows = ["source                 instances  VGPRs(max) AGPRs(max) scratch(max) spills(max) LDS_bytes(min..max) waves/SIMD(min..max)  kernel template"]
    for (src, name), ks in sorted(fam.items()):
        g = lambda f: [int(k.get(f, 0)) for k in ks]
        lds, occ = g("LDS Size [bytes/block]"), g("Occupancy [waves/SIMD]")
        rows.append(f"{src:<22} {len(ks):>9}  {max(g('VGPRs')):>10} {max(g('AGPRs')):>10} {max(g('ScratchSize [bytes/lane]')):>12} "
                    f"{max(g('VGPRs Spill')) + max(g('SGPRs Spill')):>11} {f'{min(lds)}..{max(lds)}':>19} {f'{min(occ)}..{max(occ)}':>20}  {name}")
    return "\n".join(rows) + "\n"


def _wait(procs, verbose, table):
    while procs:
        src, p = procs.pop(0)
        out, _ = p.communicate()
        table.extend(parse_resources(src, out))
        lines = [l for l in out.splitlines() if "packed-fp32-ops" not in l]
        if p.returncode != 0:
            sys.stderr.write("\n".join(lines) + "\n")
            raise RuntimeError(f"hipcc failed on {src}")
        # the remarks (three lines each) are parsed above, not echoed
        keep, in_remark = [], False
        for l in lines:
            if "-Rpass-analysis=kernel-resource-usage" in l:
                in_remark = True
                continue
            if in_remark and re.match(r"^\s*\d*\s*\|", l):
                continue
            in_remark = False
            keep.append(l)
        if verbose and keep:
            print("\n".join(keep), flush=True)


if __name__ == "__main__":
    print(build_library(verbose=True))
    if len(sys.argv) == 3 and sys.argv[1] == "--resources":
        # a copy of the per-kernel resource table (registers, scratch, LDS, occupancy) for the records
        with open(os.path.join(PKG, "_build", "kernel_resources_summary.txt")) as f, open(sys.argv[2], "w") as g:
            g.write("Resource usage of every kernel template, reported by hipcc (-Rpass-analysis=kernel-resource-usage) for gfx950;\n"
                    "extremes over the instantiations of a template (the table per instantiation is written next to the objects).\n"
                    "command: python -m paper_2209_06979_amd.build --resources <this file>\n"
                    "The build fails if a kernel of a source that issues untracked global -> LDS copies (copy16_to_lds) reports\n"
                    "scratch or spilled registers.\n\n")
            g.write(f.read())
