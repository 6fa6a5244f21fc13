"""Build libleanquant.so (gfx950) in-tree with hipcc.  `python -m paper_2407_10032_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libleanquant.so")
SOURCES = ["quantize_col128.hip", "quantize_col64.hip", "quantize_col32.hip", "api.hip", "hessian.hip",
           "cholesky.hip", "fit_grid.hip", "quantize.hip", "pack.hip", "exact.hip", "gemv.hip", "gemm_packed.hip", "seed.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    # packed-fp32 code generation is switched off for every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


_COL_HEADERS = ("lq_quantize_col.h", "lq_common.h", "lq_mfma.h")


def _newest_header(src: str) -> float:
    """Newest header the source can depend on (the column-kernel units use only three)."""
    names = _COL_HEADERS if src.startswith("quantize_col") else tuple(
        f for f in os.listdir(CSRC) if f.endswith(".h"))
    paths = [os.path.join(CSRC, f) for f in names] + [os.path.join(HERE, "..", "include", "leanquant.h")]
    return max(os.path.getmtime(p) for p in paths)


def _compile(src: str, incremental: bool = False) -> str:
    obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
    if incremental and os.path.exists(obj):
        if os.path.getmtime(obj) > max(os.path.getmtime(os.path.join(CSRC, src)), _newest_header(src)):
            return obj
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, res.stdout, res.stderr))
    return obj


def build(verbose: bool = True, incremental: bool = False) -> str:
    """Compile every source for gfx950 and link the shared library.  `incremental`
    skips objects newer than their source and all headers (developer convenience)."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, incremental), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (res.stdout, res.stderr))
    if verbose:
        print("built", LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    build(incremental="--incremental" in sys.argv)
    sys.exit(0)
