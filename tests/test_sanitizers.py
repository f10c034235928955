"""AddressSanitizer + UndefinedBehaviorSanitizer over everything that runs on the host: the C oracle on
small inputs in exactly-sized heap blocks, and the library's host side (validation, size arithmetic,
split planning, error text) through every entry point on a context without a device.  No GPU, and no GPU
sanitizer: only host code is instrumented."""
import os
import subprocess

import pytest

from paper_2605_19218_amd import build as hip_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-g", "-O1"]


def clang():
    cc = hip_build.host_clang()
    if not os.path.exists(cc):
        pytest.skip("no clang with sanitizer run-times")
    return cc


def run_clean(exe):
    res = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    text = res.stdout + res.stderr
    assert res.returncode == 0, text
    assert "runtime error" not in text and "Sanitizer" not in text, text
    return res.stdout


def test_oracle_c_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.run([clang(), "-std=c99", "-Wall", "-Wextra", "-ffp-contract=off"] + SAN +
                   [os.path.join(ROOT, "tests", "c_abi", "oracle_san.c"), os.path.join(ROOT, "oracle", "rotatek_oracle.c"),
                    "-o", exe, "-lm"], check=True)
    assert "ran clean" in run_clean(exe)


def test_library_host_side_under_sanitizers(tmp_path):
    cc = clang()
    lib = hip_build.build_host_sanitized(str(tmp_path))
    libdir = os.path.dirname(lib)
    for src in ("host_sweep.c", "host_calls.c"):
        exe = str(tmp_path / src[:-2])
        subprocess.run([cc, "-std=c99", "-Wall", "-Wextra"] + SAN +
                       ["-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "c_abi", src), "-o", exe,
                        "-L", libdir, "-lrotatek_san", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"], check=True)
        out = run_clean(exe)
        assert ("checks passed" in out) if src == "host_sweep.c" else ("device" in out)
