"""Builds libcachefocus.so in-tree with hipcc for gfx950.

Usage: python -m paper_2502_11101_amd.build
"""

from __future__ import annotations

import json
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcachefocus.so")
SOURCES = ["cf_api.hip", "cf_reposition.hip", "cf_attn_generic.hip", "cf_attn_mfma.hip", "cf_attn_reduce.hip", "cf_select.hip", "cf_calibrate.hip"]
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Rpass-analysis=kernel-resource-usage",
]
RESOURCES = os.path.join(HERE, "kernel_resources.json")
# kernels on the hot path that must keep everything in registers: a spill to scratch memory there
# (a few lines of source can tip the register allocator over) costs far more than any tuning gains
NO_SCRATCH = ("attn_tile_kernel", "attn_pipe_kernel", "attn_combine_kernel", "layer_epilogue_kernel", "reposition_kernel",
              "assemble_kernel")


def build(verbose: bool = True, jobs: int = 8) -> str:
    """Compile every translation unit and link the shared library; returns its path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    procs = []
    objs = []
    usage = {}
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc, *FLAGS, *inc, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _wait(procs, verbose, usage)
    _wait(procs, verbose, usage)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    with open(RESOURCES, "w") as f:
        json.dump(usage, f, indent=1, sort_keys=True)
    spilling = sorted(k for k, u in usage.items() if u.get("scratch_bytes", 0) > 0 and any(n in k for n in NO_SCRATCH))
    if spilling:
        raise RuntimeError("hot-path kernels spill registers to scratch memory: " +
                           ", ".join(f"{k} ({usage[k]['scratch_bytes']} B/lane)" for k in spilling))
    return LIB


_FIELDS = {"VGPRs": "vgprs", "AGPRs": "agprs", "ScratchSize [bytes/lane]": "scratch_bytes",
           "Occupancy [waves/SIMD]": "waves_per_simd", "LDS Size [bytes/block]": "lds_bytes", "TotalSGPRs": "sgprs"}


def _collect_usage(out: str, usage: dict) -> list:
    """Takes the compiler's per-kernel resource remarks out of its output (into `usage`, keyed by the
    demangled kernel name where c++filt knows it) and returns the remaining lines."""
    rest, current = [], None
    for line in out.splitlines():
        if "-Rpass-analysis=kernel-resource-usage" not in line:
            if not (current is not None and re.match(r"^\s*(\d+\s*\||\||\^)", line)):      # the source excerpt under a remark
                rest.append(line)
            continue
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            current = usage.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z][^:]*): (\S+)", line)
        if m and current is not None and m.group(1) in _FIELDS:
            try:
                current[_FIELDS[m.group(1)]] = int(m.group(2))
            except ValueError:
                pass
    return rest


def _wait(procs, verbose, usage):
    failed = []
    for src, p in procs:
        out, _ = p.communicate()
        lines = [l for l in _collect_usage(out, usage) if "packed-fp32-ops" not in l]
        if verbose and lines:
            print("\n".join(lines), flush=True)
        if p.returncode != 0:
            failed.append(src)
    procs.clear()
    if failed:
        raise RuntimeError(f"hipcc failed for {failed}")


if __name__ == "__main__":
    build()
    print("built", LIB)
