"""Build libsgap.so (HIP, gfx950) in-tree with hipcc.  No GPU is needed."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsgap.so")
SOURCES = [
    "sgap_api.hip", "sgap_row_split.hip", "sgap_row_split_partial.hip", "sgap_sddmm.hip", "sgap_mttkrp.hip", "sgap_panels.hip", "sgap_wave_rows.hip", "sgap_reorder.hip", "sgap_mttkrp_nnz.hip",
    "sgap_nnz_parallel.hip", "sgap_nnz_parallel_g1.hip", "sgap_nnz_parallel_g2.hip",
    "sgap_nnz_parallel_g4_16.hip", "sgap_nnz_parallel_g8_32_64.hip",
    "sgap_nnz_serial.hip", "sgap_nnz_serial_lc1_2.hip", "sgap_nnz_serial_lc4_8.hip",
    "sgap_nnz_serial_lc16_32.hip", "sgap_nnz_serial_lc64.hip",
]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stderr}")
    return obj


def build_library(jobs: int = 8) -> str:
    """Compile every source and link the shared library; always rebuilds."""
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    return LIB


MICROBENCH = os.path.join(HERE, "microbench")


def build_microbenchmarks() -> list[str]:
    """Compile the standalone microbenchmarks (microbench/*.hip -> microbench/bin/)."""
    out_dir = os.path.join(MICROBENCH, "bin")
    os.makedirs(out_dir, exist_ok=True)
    built = []
    for src in sorted(f for f in os.listdir(MICROBENCH) if f.endswith(".hip")):
        exe = os.path.join(out_dir, src[:-4])
        cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-munsafe-fp-atomics", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-Wno-unused-command-line-argument", os.path.join(MICROBENCH, src), "-o", exe]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{r.stderr}")
        built.append(exe)
    return built


if __name__ == "__main__":
    import sys

    print(build_library())
    if "--microbench" in sys.argv[1:]:
        print("\n".join(build_microbenchmarks()))
