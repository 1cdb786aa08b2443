"""Build libskrull_attn.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libskrull_attn.so")
SOURCES = ["api.hip", "plan.hip", "fwd.hip", "bwd.hip", "probe.hip", "dacp.cpp", "gds.cpp"]
# packed fp32 VALU ops are switched off for all device code
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-I" + os.path.join(ROOT, "include"),
         "-I" + CSRC, "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Wno-inline-asm"]
# further compiler flags for experiments (space separated), e.g. SKRULL_EXTRA_FLAGS="-mllvm -align-loops=64"
FLAGS += os.environ.get("SKRULL_EXTRA_FLAGS", "").split()


def _compile(src: str) -> str:
    """Compile one source.  The compiler's per-kernel resource remarks are
    parsed and the build fails if any kernel uses scratch memory: register
    spills cost bandwidth in the hot loops, and a partially spilled MFMA
    operand tuple has been seen to be reloaded incompletely by this compiler
    (wrong results), so spilling kernels are not allowed in the library."""
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    r = subprocess.run(["hipcc", *FLAGS, "-Rpass-analysis=kernel-resource-usage", "-c",
                        os.path.join(CSRC, src), "-o", obj], stderr=subprocess.PIPE, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr}")
    name, report = None, []
    for line in r.stderr.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and name:
            report.append((name, int(m.group(1))))
            if int(m.group(1)) != 0:
                raise RuntimeError(f"{src}: kernel {name} spills {m.group(1)} bytes/lane to scratch")
    if not os.environ.get("SKRULL_QUIET"):
        for line in r.stderr.splitlines():
            if "error" in line or ("warning" in line and "packed-fp32" not in line):
                print(line)
    return obj


def build_library(jobs: int = 4) -> str:
    """Compile every HIP source and link the shared library; returns its path."""
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    print(build_library())
