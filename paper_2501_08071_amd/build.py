"""Compile the HIP sources into the in-tree C-ABI shared library (gfx950 only)."""
from __future__ import annotations

import os
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libattn_gfx950.so")
SOURCES = ["attn_fwd_gfx950.hip", "attn_fwd_rows64_gfx950.hip", "attn_api.cpp", "rowops_gfx950.hip", "rowops_api.cpp",
           "gemm_gfx950.hip", "gemm_api.cpp", "probe_gfx950.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# packed-fp32 VALU forms are switched off for all device code
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument", "-Wno-inline-asm"]
# Per source.  The kernel whose wavefronts own the whole register file (one per SIMD) asks the compiler to keep matrix
# results where vector instructions can read them (the scores are consumed by the vector pipe); left to its own
# heuristic it puts every matrix result of such a kernel into accumulation registers and copies the scores out
# element by element.
SOURCE_FLAGS = {"attn_fwd_rows64_gfx950.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}
NOISE = "is not a recognized feature for this target"


def _run(cmd):
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if NOISE not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{' '.join(cmd)}\n{err}")
    return err


def build_lib(extra_flags=(), out: str = LIB, verbose: bool = False, jobs: int = 4) -> str:
    """Every source to an object of its own (with its own flags), then one link."""
    tmp = tempfile.mkdtemp(prefix="attn_build_")
    try:
        def compile_one(src):
            obj = os.path.join(tmp, src + ".o")
            cmd = [HIPCC, *FLAGS, *SOURCE_FLAGS.get(src, ()), *extra_flags, "-c", "-x", "hip", os.path.join(CSRC, src), "-o", obj]
            return obj, _run(cmd)

        with ThreadPoolExecutor(max_workers=jobs) as ex:
            done = list(ex.map(compile_one, SOURCES))
        err = "".join(e for _, e in done)
        err += _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *[o for o, _ in done], "-o", out])
        if verbose and err.strip():
            print(err)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return out


def lib_is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(HERE, "..", "include", h) for h in ("attn.h", "rowops.h", "gemm.h", "probe.h")]
    return any(os.path.getmtime(d) > t for d in deps)


if __name__ == "__main__":
    print(build_lib(verbose=True))
