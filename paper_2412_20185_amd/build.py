"""Builds libdecdec.so (HIP kernels + C ABI) for gfx950, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdecdec.so")
SOURCES = ("api.hip", "gemv.hip", "select.hip", "select_bucket.hip", "fetch.hip", "fused.hip", "accumulate.hip", "quantize.hip",
           "residual_quantize.hip")
FLAGS = ("-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument")


def _run(cmd) -> str:
    res = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
    return out


def build(verbose: bool = False, jobs: int | None = None) -> str:
    """Compiles every source to an object file (in parallel), links them into the shared library and
    replaces the old library only when all of that has succeeded."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    inc = os.path.join(os.path.dirname(HERE), "include")
    jobs = jobs or min(len(SOURCES), max(1, min(os.cpu_count() or 1, 8)))
    with tempfile.TemporaryDirectory(prefix="decdec_build_") as tmp:
        def compile_one(src: str) -> str:
            obj = os.path.join(tmp, src + ".o")
            return _run([hipcc, *FLAGS, "-I", inc, "-c", os.path.join(CSRC, src), "-o", obj])

        with ThreadPoolExecutor(max_workers=jobs) as pool:
            logs = list(pool.map(compile_one, SOURCES))
        logs.append(_run([hipcc, "--offload-arch=gfx950", "-fPIC", "-shared",
                          *[os.path.join(tmp, s + ".o") for s in SOURCES], "-o", LIB + ".tmp"]))
    os.replace(LIB + ".tmp", LIB)
    out = "\n".join(l for l in logs if l.strip())
    if verbose and out.strip():
        print(out)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
