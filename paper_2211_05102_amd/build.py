"""Builds libpalmdecode.so (gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpalmdecode.so")
SOURCES = ["qgemm.hip", "wgemm.hip", "attention.hip", "pointwise.hip", "sampler.hip", "probe.hip", "api.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    subprocess.run([HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj], check=True,
                   stderr=subprocess.DEVNULL if os.environ.get("PD_QUIET") else None)
    return obj


def build() -> str:
    """Compiles every source and links the shared library; always recompiles."""
    with ThreadPoolExecutor(max_workers=7) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    print(build())
