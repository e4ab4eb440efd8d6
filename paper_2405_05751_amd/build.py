"""Compile the HIP sources under csrc/ into paper_2405_05751_amd/librmsnl.so for gfx950.

hipcc cross-compiles without a GPU.  Objects are built in parallel into csrc/_build/ and
linked into one shared library that exports only the C ABI of include/rmsnl.h.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "librmsnl.so")
SOURCES = ["api.hip", "naive.hip", "gemv.hip", "skinny.hip", "tile.hip", "f32.hip", "ntrans.hip", "qkattn.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    # no packed-fp32 VALU forms: scalar fp32 code must stay scalar on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # leading scalar kernel arguments arrive in registers (preloaded by the dispatcher) instead of by a load
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def _compile(src: str, extra, objdir: str = OBJ) -> str:
    out = os.path.join(objdir, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                     if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{msgs}")
    if msgs:
        print(msgs, file=sys.stderr)
    return out


def build(force: bool = True, extra_flags=(), out: str = LIB) -> str:
    """Compile and link; `out` and `extra_flags` let experiments build side-by-side variants."""
    if out != LIB:
        return _link(out, extra_flags, os.path.join(OBJ, os.path.basename(out) + ".d"))
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    deps = srcs + [os.path.join(CSRC, "common.hpp"), os.path.join(CSRC, "splitk.hpp"), os.path.join(HERE, "..", "include", "rmsnl.h")]
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    return _link(LIB, extra_flags, OBJ)


def _link(out: str, extra_flags, objdir: str) -> str:
    os.makedirs(objdir, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, list(extra_flags), objdir), SOURCES))
    tmp = out + f".tmp{os.getpid()}"
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]
    subprocess.run(cmd, check=True)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    flags = [a for a in sys.argv[1:] if not a.startswith("--out=")]
    outs = [a[6:] for a in sys.argv[1:] if a.startswith("--out=")]
    print(build(extra_flags=flags, out=os.path.abspath(outs[0]) if outs else LIB))
