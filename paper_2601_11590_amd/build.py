"""Build ``libepd_encode.so`` (hand-written HIP kernels + the C ABI) for gfx950 with hipcc.

The library is built in-tree, next to this file, so that it travels with the source tree.
hipcc cross-compiles for gfx950 without a GPU being present.
"""

from __future__ import annotations

import hashlib
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libepd_encode.so")
STAMP = LIB + ".hash"         # source_hash() of the sources LIB was built from
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["epd_api.hip", "plan_norm.hip", "preprocess.hip", "mm_store.hip", "probe.hip", "kernels_f32.hip", "gemm_bf16.hip", "attn_bf16.hip"]

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


def source_hash(extra_flags=()) -> str:
    """SHA-256 over everything the binary depends on: every file under csrc/, the public
    header, the compiler flags and the source list."""
    h = hashlib.sha256()
    files = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC))
    files.append(os.path.join(os.path.dirname(HERE), "include", "epd_encode.h"))
    for path in files:
        h.update(os.path.basename(path).encode() + b"\0")
        with open(path, "rb") as f:
            h.update(f.read())
        h.update(b"\0")
    h.update(repr((SOURCES, FLAGS, tuple(extra_flags))).encode())
    return h.hexdigest()


def built_hash() -> str:
    """The hash stored next to the library when it was built ('' if there is none)."""
    try:
        with open(STAMP) as f:
            return f.read().strip()
    except OSError:
        return ""


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every source and link the shared library.  Returns its path."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    if os.path.exists(STAMP):
        os.remove(STAMP)
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
    with open(STAMP, "w") as f:
        f.write(source_hash(extra_flags) + "\n")
    return LIB


def library_path(build_if_missing: bool = True) -> str:
    """Path of the built library.  The library is tied to its sources by the hash stored next
    to it: a missing library, a missing stamp or a stamp that differs from the hash of the
    sources as they stand (an edit without a rebuild) makes this build again, loudly, so that
    tests and benchmarks never run a binary that is not the committed source."""
    have = os.path.exists(LIB)
    stale = have and built_hash() != source_hash()
    if not have or stale:
        if not build_if_missing:
            raise FileNotFoundError(LIB if not have else LIB + " is older than its sources")
        print("[epd build] %s: building libepd_encode.so now (hipcc, about two minutes)"
              % ("the library is STALE against csrc/" if stale else "no library yet"), file=sys.stderr, flush=True)
        build()
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
