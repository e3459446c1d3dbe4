"""Builds libzeda.so (HIP, gfx950 only) in-tree with hipcc.  `python -m paper_2605_18643_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
LIB = os.path.join(LIB_DIR, "libzeda.so")
SOURCES = ["zeda_api.hip", "zeda_route.hip", "zeda_dispatch.hip", "zeda_ffn.hip", "zeda_combine.hip", "zeda_stack.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # packed fp32 instructions are switched off for all device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _run(cmd, verbose: bool) -> None:
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the device-only target feature and says so once per file
    err = "\n".join(l for l in proc.stderr.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        sys.stderr.write(err + "\n")
        raise RuntimeError("hipcc failed building libzeda.so")
    if verbose and err.strip():
        print(err)


def build(verbose: bool = False) -> str:
    """Compiles every source (one hipcc per file, side by side) and links lib/libzeda.so.  Always compiles."""
    os.makedirs(LIB_DIR, exist_ok=True)
    with tempfile.TemporaryDirectory(prefix="zeda_build_") as tmp:
        objs = [os.path.join(tmp, s.replace(".hip", ".o")) for s in SOURCES]
        with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
            list(pool.map(lambda so: _run(["hipcc", *FLAGS, "-c", os.path.join(CSRC, so[0]), "-o", so[1]], verbose),
                          zip(SOURCES, objs)))
        _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], verbose)
    return LIB


def device_isa(source: str, out_path: str) -> str:
    """Device-side ISA text (hipcc -S) of one of SOURCES, for lds_wait_check."""
    cmd = ["hipcc", *FLAGS, "-S", "--cuda-device-only", os.path.join(CSRC, source), "-o", out_path]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        sys.stderr.write(proc.stderr)
        raise RuntimeError(f"hipcc -S failed on {source}")
    return out_path


if __name__ == "__main__":
    print(build(verbose=True))
