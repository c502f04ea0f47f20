"""Build liblcd.so (HIP, gfx950 only) in-tree with hipcc.  No JIT, no torch extension."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
CSRC = PKG / "csrc"
LIB = PKG / "liblcd.so"
BUILD = ROOT / "_build"

SOURCES = ["lcd_host.cpp", "lcd_pack.hip", "lcd_gemv.hip", "lcd_gemm.hip", "lcd_cluster.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    f"-I{ROOT / 'include'}", f"-I{CSRC}",
]


# lcd_gemm.hip keeps its accumulators in fixed AGPRs through inline assembly: the compiler must not
# use AGPRs as spill space there.
# lcd_gemv.hip: the decode kernels' eight leading scalar arguments (the table of first workgroups) are
# preloaded into scalar registers at wave start instead of being read from the argument segment.
EXTRA = {"lcd_gemm.hip": ["-mllvm", "-amdgpu-spill-vgpr-to-agpr=0"],
         "lcd_gemv.hip": ["-mllvm", "-amdgpu-kernarg-preload-count=8"]}


def _compile(src: str, keep_asm: bool) -> Path:
    obj = BUILD / (src.rsplit(".", 1)[0] + ".o")
    cmd = [HIPCC, *FLAGS, *EXTRA.get(src, []), "-c", str(CSRC / src), "-o", str(obj)]
    if keep_asm and src.endswith(".hip"):
        cmd += ["-save-temps=obj"]
    subprocess.check_call(cmd, cwd=str(BUILD), stderr=subprocess.DEVNULL if not os.environ.get("LCD_BUILD_VERBOSE") else None)
    return obj


def build_library(keep_asm: bool = False) -> Path:
    """Compile every source and link paper_2506_12038_amd/liblcd.so."""
    BUILD.mkdir(exist_ok=True)
    srcs = [s for s in SOURCES if (CSRC / s).exists()]
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda s: _compile(s, keep_asm), srcs))
    tmp = LIB.with_suffix(".so.tmp%d" % os.getpid())
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *map(str, objs), "-o", str(tmp)])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(keep_asm=bool(os.environ.get("LCD_KEEP_ASM"))))
