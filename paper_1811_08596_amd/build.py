"""Builds libfftsp.so (the HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfftsp.so")
SOURCES = ["fft.hip", "fused.hip", "codec.hip", "api.hip", "prof.hip"]
HEADERS = [os.path.join(CSRC, "internal.h"), os.path.join(CSRC, "fft_core.h"), os.path.join(CSRC, "twiddle_table.h"), os.path.join(os.path.dirname(HERE), "include", "fftsp.h")]

# no fast-math: twiddles, keys and the split must round the same way on every launch
HIPCC_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-fconstexpr-steps=50000000",
]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = ["hipcc", *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    errs = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr}")
    if errs:
        print(errs)
    return obj


def build_lib(force: bool = True) -> str:
    """Compile every HIP source and link the shared library; returns its path."""
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    print(build_lib())
