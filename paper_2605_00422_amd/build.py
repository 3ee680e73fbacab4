"""Build libbwla.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libbwla.so")
SOURCES = ["api.hip", "pack.hip", "rotate_quant.hip", "gemm_decode.hip", "gemm_decode_bs.hip", "gemm_prefill.hip", "psp_prefill.hip", "decode_layer.hip",
           "probe.hip", "rotate_planes.hip",
           "quantizer_api.hip", "quantizer_gemm.hip", "quantizer_rows.hip", "quantizer_jacobi.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


# Per-file flags.  decode_layer.hip: the first 14 dwords of its kernels' arguments (seven pointers)
# are preloaded into SGPRs when a wavefront starts, instead of being fetched by the kernel.
FILE_FLAGS = {"decode_layer.hip": ["-mllvm", "-amdgpu-kernarg-preload-count=14"]}


def _compile(src: str, extra: list[str]) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, *FILE_FLAGS.get(src, []), *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines()
                    if "not a recognized feature for this target" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_library(extra_flags: list[str] | None = None, jobs: int = 6) -> str:
    extra = list(extra_flags or [])
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(sys.argv[1:]))
