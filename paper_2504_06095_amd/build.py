"""Builds libntp.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libntp.so")

SOURCES = ["ntp_plan.cpp", "ntp_handle.hip", "ntp_layers.cpp", "ntp_timing.cpp", "ntp_gemm.hip", "ntp_gemm_nt.hip", "ntp_gemm_nn.hip",
           "ntp_gemm_tn.hip", "ntp_gemm_pp_nt.hip", "ntp_gemm_pp_nn.hip", "ntp_gemm_pp_tn.hip", "ntp_reshard.hip", "ntp_attn_core.hip", "ntp_probe.hip"]

# -packed-fp32-ops is switched off: the compiler must not form packed fp32 VALU ops.
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _run(cmd: list[str]) -> str:
    res = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(ln for ln in (res.stdout + res.stderr).splitlines() if "not a recognized feature" not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + out)
    return out


def build_library(verbose: bool = False, jobs: int | None = None) -> str:
    """Compile every source (in parallel, one hipcc per file) and link the shared library.  Always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    jobs = jobs or min(len(SOURCES), int(os.environ.get("MAX_JOBS", "8")), os.cpu_count() or 8)
    with tempfile.TemporaryDirectory(prefix="ntp_build_") as tmp:
        def compile_one(src: str) -> tuple[str, str]:
            obj = os.path.join(tmp, src + ".o")
            cmd = [hipcc, *HIP_FLAGS, "-c", "-I", os.path.join(ROOT, "include"), "-I", CSRC, os.path.join(CSRC, src),
                   "-o", obj]
            return obj, _run(cmd)
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            results = list(pool.map(compile_one, SOURCES))
        out = "\n".join(o for _, o in results if o.strip())
        out += _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *[obj for obj, _ in results], "-o", LIB_PATH])
    if verbose and out.strip():
        print(out)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
