"""Builds libsvgear.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libsvgear.so")
SOURCES = ["api.hip", "permute.hip", "kmeans.hip", "probe.hip", "route.hip", "attention.hip", "attention_bf16.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    *os.environ.get("SVGEAR_HIPCC_FLAGS", "").split(),  # extra flags for experiments, e.g. -DNAME=value
]


# host code only (argument checks, launch logic) under AddressSanitizer / UBSan; device code is unchanged
HOST_SANITIZE_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                       "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def _compile(src: str, objdir: str, extra=()) -> str:
    obj = os.path.join(objdir, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    return obj


def build(verbose: bool = False, lib: str = LIB, objdir: str | None = None, host_sanitize: bool = False) -> str:
    """Compiles every source and links the shared library; always rebuilds. host_sanitize=True
    builds a copy whose HOST code runs under AddressSanitizer and UBSan (for a CPU test binary;
    give it its own `lib` and `objdir`)."""
    objdir = os.path.join(_HERE, "_build") if objdir is None else objdir
    os.makedirs(objdir, exist_ok=True)
    extra = HOST_SANITIZE_FLAGS if host_sanitize else ()
    with ThreadPoolExecutor(max_workers=min(6, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, objdir, extra), SOURCES))
    link_extra = ["-fsanitize=address", "-fsanitize=undefined"] if host_sanitize else []
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *link_extra, *objs, "-o", lib]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    build(verbose=True)
