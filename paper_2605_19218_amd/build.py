"""Compile the HIP kernels and the C ABI into paper_2605_19218_amd/librotatek.so (gfx950)."""
from __future__ import annotations

import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

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


def _report_scratch(stderr_lines) -> None:
    """A kernel that spills registers to scratch memory runs an order of magnitude slower: say so loudly."""
    name = None
    for l in stderr_lines:
        if "Function Name:" in l:
            name = l.split("Function Name:")[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in l:
            n = int(l.split("ScratchSize [bytes/lane]:")[1].split("[")[0])
            if n > 0:
                print(f"WARNING: kernel {name} uses {n} bytes/lane of scratch (register spills)")


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless.  The resource
    # remarks come with source-context lines ("  105 | {" / "      | ^"): keep only real diagnostics.
    lines = [l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l]
    remarks = [l for l in lines if "-Rpass-analysis=kernel-resource-usage" in l]
    ctx = re.compile(r"^\s*\d*\s*\|")
    err = "\n".join(l for l in lines if "-Rpass-analysis=kernel-resource-usage" not in l and not ctx.match(l)
                    and "remarks generated" not in l and "warning generated" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return remarks


def build(verbose: bool = False) -> str:
    """Compile every source to an object (in parallel) and link librotatek.so."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    common = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              "-Wno-unused-command-line-argument", "-Rpass-analysis=kernel-resource-usage",
              "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    objs = [os.path.join(objdir, s.replace(".hip", ".o")) for s in SOURCES]
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        jobs = [ex.submit(_run, common + ["-c", os.path.join(CSRC, s), "-o", o], verbose) for s, o in zip(SOURCES, objs)]
        remarks = [r for j in jobs for r in j.result()]
    _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, verbose)
    _report_scratch(remarks)
    return LIB


def build_host_sanitized(outdir: str) -> str:
    """A second copy of the library, in `outdir`, whose HOST code is built with AddressSanitizer and
    UndefinedBehaviorSanitizer (the device code is compiled unoptimised: it is never run).  For host-only
    runs on a context without a device; the GPU sanitizers are not used."""
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    common = [hipcc(), "--offload-arch=gfx950", "-O1", "-Xarch_device", "-O0", "-g", "-std=c++17", "-fPIC",
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
              "-I", os.path.join(ROOT, "include"), "-I", CSRC] + san
    objs = [os.path.join(outdir, s.replace(".hip", ".o")) for s in SOURCES]
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        jobs = [ex.submit(_run, common + ["-c", os.path.join(CSRC, s), "-o", o], False) for s, o in zip(SOURCES, objs)]
        for j in jobs:
            j.result()
    lib = os.path.join(outdir, "librotatek_san.so")
    _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC"] + san[:4] + ["-o", lib] + objs, False)
    return lib


def host_clang() -> str:
    """The C compiler that matches the sanitizer run-time of build_host_sanitized (ROCm's clang)."""
    return os.path.join(os.path.dirname(os.path.dirname(os.path.realpath(hipcc()))), "lib", "llvm", "bin", "clang")


if __name__ == "__main__":
    print(build(verbose=True))
