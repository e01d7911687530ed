"""Compile the HIP library for gfx950 with hipcc (cross-compiles without a GPU).

Every source is compiled to an object of its own, several at a time, then linked; the objects live
in ``_build/`` next to this file.  The compiler's per-kernel resource remarks are collected into
``_build/resources.txt`` (registers, scratch bytes per lane, LDS per kernel): the place to look when a change
to the streaming attention kernel makes an instance an order of magnitude slower, which is what happens when
its tile ring or accumulators no longer fit the register file.  (The instances with four and five row blocks
spill some values at entry that only the end of a unit reloads; their tile bodies touch no scratch.)
"""
from __future__ import annotations

import concurrent.futures
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libspecverify.so")
# the per-grouping attention units take longest: start them first
SOURCES = ["attn_mfma_g8.hip", "attn_mfma_g4.hip", "attn_mfma_g2.hip", "attn_mfma_g1.hip", "accept.hip", "accept_tree.hip", "accept_static.hip", "api.hip",
           "attn_mfma.hip", "attn_generic.hip", "kvcache.hip", "validate.hip", "depth_controller.cpp", "router.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Rpass-analysis=kernel-resource-usage",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]
# the host pass reports that it does not know the packed-fp32 feature; that line is noise
NOISE = "is not a recognized feature for this target"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    lines = [l for l in res.stderr.splitlines() if NOISE not in l]
    # what is left for the log: everything but the resource remarks with their "included from" headers and
    # source excerpts (the lines between a remark and the next diagnostic)
    kept, in_remark = [], False
    for l in lines:
        if "remark:" in l:
            in_remark = True
            while kept and kept[-1].startswith("In file included from"):
                kept.pop()
            continue
        if in_remark and (l.startswith(" ") or l.startswith("In file included from") or not l.strip()):
            if l.startswith("In file included from"):
                kept.append(l)   # may belong to a real diagnostic that follows; dropped again if a remark does
                in_remark = False
            continue
        in_remark = False
        kept.append(l)
    while kept and kept[-1].startswith("In file included from"):
        kept.pop()
    err = "\n".join(kept)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + err)
    return err, _resources(lines)


def _resources(lines):
    """{mangled kernel name: {"VGPRs": n, "AGPRs": n, "ScratchSize": bytes per lane, "LDS Size": bytes}} from the remarks."""
    out, cur = {}, None
    for l in lines:
        m = re.search(r"remark: .*Function Name: (\S+)", l)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark: .*?\s(VGPRs|AGPRs|ScratchSize|LDS Size)[^:]*: (\d+)", l)
        if m and cur is not None:
            cur.setdefault(m.group(1), int(m.group(2)))
    return out


def build(verbose: bool = False, jobs: int = 0) -> str:
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or min(len(SOURCES), max(1, (os.cpu_count() or 2) - 1), 8)
    objects = [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
        futs = [pool.submit(_run, ["hipcc", *FLAGS, "-c", os.path.join(CSRC, s), "-o", o], verbose)
                for s, o in zip(SOURCES, objects)]
        results = [f.result() for f in futs]   # raises the first failure
    warnings = [r[0] for r in results]
    report = {}
    for r in results:
        report.update(r[1])
    with open(os.path.join(OBJ, "resources.txt"), "w") as f:
        for name in sorted(report):
            f.write(name + " " + " ".join(f"{k.replace(' ', '_')}={v}" for k, v in report[name].items()) + "\n")
    warnings.append(_run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objects], verbose)[0])
    if verbose:
        for w in warnings:
            if w.strip():
                print(w, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
