"""Builds librealb.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "librealb.so")
SOURCES = ["context.hip", "quantize.hip", "route_stats.hip", "permute.hip", "ffn.hip", "combine.hip", "layer.hip", "nvfp4.hip"]
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-Rpass-analysis=kernel-resource-usage",      # per-kernel register / scratch report, checked below
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def kernel_usage(stderr: str) -> dict:
    """Parses hipcc's kernel-resource-usage remarks: {kernel: {vgprs, scratch, vgpr_spill}}."""
    import re
    usage, cur = {}, None
    for l in stderr.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", l)
        if m:
            cur = usage.setdefault(m.group(1), {})
            continue
        if cur is None:
            continue
        for key, pat in (("vgprs", r"remark:\s+VGPRs: (\d+)"), ("scratch", r"ScratchSize \[bytes/lane\]: (\d+)"),
                         ("vgpr_spill", r"VGPRs Spill: (\d+)")):
            m = re.search(pat, l)
            if m:
                cur[key] = int(m.group(1))
    return usage


def build(verbose: bool = False) -> str:
    """Compiles every HIP source into librealb.so; always recompiles."""
    cmd = [hipcc(), *HIPCC_FLAGS, *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB_PATH + ".tmp"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    usage = kernel_usage(res.stderr)
    noise = ("is not a recognized feature for this target", "-Rpass-analysis=kernel-resource-usage")
    lines, skip = [], 0
    for l in res.stderr.splitlines():                # drop the resource remarks and their two source-quote lines
        if "-Rpass-analysis=kernel-resource-usage" in l:
            skip = 2
            continue
        if skip and (l.lstrip().startswith("|") or l.lstrip()[:1].isdigit()):
            skip -= 1
            continue
        skip = 0
        if not any(n in l for n in noise):
            lines.append(l)
    err = "\n".join(lines)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    # A kernel that spills is a performance bug here (a scratch reload waits for every outstanding
    # memory transfer of the wave): refuse to ship it silently.
    spilled = {k: u for k, u in usage.items() if u.get("scratch", 0) or u.get("vgpr_spill", 0)}
    if spilled:
        raise RuntimeError("kernels with register spills / scratch: " + ", ".join(f"{k} {u}" for k, u in spilled.items()))
    if verbose and err.strip():
        print(err, file=sys.stderr)
    os.replace(LIB_PATH + ".tmp", LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
