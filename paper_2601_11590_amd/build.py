"""Build ``libepd_encode.so`` (hand-written HIP kernels + the C ABI) for gfx950 with hipcc.

The library is built in-tree, next to this file, so that it travels with the source tree.
hipcc cross-compiles for gfx950 without a GPU being present.
"""

from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libepd_encode.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["epd_api.hip", "plan_norm.hip", "preprocess.hip", "mm_store.hip", "kernels_f32.hip", "gemm_bf16.hip", "attn_bf16.hip"]

# packed fp32 instructions are switched off for every kernel (hipcc -O3 would otherwise form
# them from ordinary float code)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Wno-option-ignored"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), r.stdout))
    return r.stdout


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every source and link the shared library.  Returns its path."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc = _hipcc()
    objs = [os.path.join(OBJ_DIR, s.replace(".hip", ".o")) for s in SOURCES]

    def one(pair):
        src, obj = pair
        out = _run([hipcc, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj])
        if verbose and out.strip():
            print(out)
        return obj

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), 8)) as ex:
        list(ex.map(one, zip(SOURCES, objs)))
    # the kernels that wait for inline LDS reads by hand: prove on the generated code that the
    # compiler moved no register while a read into it was pending (see check_lds_waits.py)
    from . import check_lds_waits
    check_lds_waits.check_sources(hipcc, [*FLAGS, *extra_flags],
                                  [os.path.join(CSRC, s) for s in ("gemm_bf16.hip", "attn_bf16.hip")])
    out = _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    if verbose and out.strip():
        print(out)
    return LIB


def library_path(build_if_missing: bool = True) -> str:
    """Path of the built library; builds it once if nothing has been built yet."""
    if not os.path.exists(LIB):
        if not build_if_missing:
            raise FileNotFoundError(LIB)
        build()
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
