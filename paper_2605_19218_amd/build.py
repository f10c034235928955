"""Compile the HIP kernels and the C ABI into paper_2605_19218_amd/librotatek.so (gfx950)."""
from __future__ import annotations

import os
import re
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librotatek.so")
SOURCES = ["rk_api.hip", "rk_fit.hip", "rk_compress.hip", "rk_decode.hip"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def build(verbose: bool = False) -> str:
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", "-Rpass-analysis=kernel-resource-usage",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    lines = [l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l]
    remarks = [l for l in lines if "-Rpass-analysis=kernel-resource-usage" in l]
    # (the remarks come with source-context lines "  105 | {" / "      | ^": drop those as well)
    ctx = re.compile(r"^\s*\d*\s*\|")
    err = "\n".join(l for l in lines if "-Rpass-analysis=kernel-resource-usage" not in l and not ctx.match(l)
                    and "remarks generated" not in l and "warning generated" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    # a kernel that spills registers to scratch memory runs an order of magnitude slower: say so loudly
    name = None
    for l in remarks:
        if "Function Name:" in l:
            name = l.split("Function Name:")[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in l:
            n = int(l.split("ScratchSize [bytes/lane]:")[1].split("[")[0])
            if n > 0:
                print(f"WARNING: kernel {name} uses {n} bytes/lane of scratch (register spills)")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
