"""Build libxl.so (HIP kernels + host planner + C ABI) for gfx950 with hipcc.

Run as `python -m paper_2007_06000_amd.build`; the library lands next to this
file so that it travels with the source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libxl.so")
# (source, object name, extra defines): kernels.hip is compiled twice, the split-bf16 variants on their own
SOURCES = [("kernels.hip", "kernels", []), ("kernels.hip", "kernels_b3", ["-DXL_TU_B3"]),
           ("plan.cpp", "plan", []), ("api.cpp", "api", []), ("static_run.hip", "static_run", [])]
HEADERS = [os.path.join(CSRC, "xl_internal.h"), os.path.join(CSRC, "plan.h"), os.path.join(CSRC, "thin_conv.h"),
           os.path.join(ROOT, "include", "xl.h")]

# packed-fp32 instructions are switched off for all device code
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
               "-Wno-cuda-compat", "-Wno-pass-failed",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _filter(stderr: str) -> str:
    keep = [ln for ln in stderr.splitlines() if "packed-fp32-ops" not in ln]
    return "\n".join(keep)


def _compile(item, force: bool) -> str:
    src, name, defines = item
    obj = os.path.join(OBJ, name + ".o")
    path = os.path.join(CSRC, src)
    newest = max(os.path.getmtime(p) for p in [path] + HEADERS)
    if not force and os.path.exists(obj) and os.path.getmtime(obj) >= newest:
        return obj
    cmd = [_hipcc()] + HIPCC_FLAGS + defines + ["-x", "hip", "-c", path, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    msg = _filter(r.stderr)
    if msg.strip():
        sys.stderr.write(msg + "\n")
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}")
    return obj


def build(force: bool = False, verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            sys.stderr.write(_filter(r.stderr) + "\n")
            raise RuntimeError("link failed")
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(force="--force" in sys.argv)
