"""Build libaif.so (HIP kernels + C ABI) for gfx950, in-tree.

    python -m paper_2511_12934_amd.build [--force]
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libaif.so")
# measurement tooling, a library of its own: the MFMA-loop and copy calibrators and the attention loop of profiling/peaks.py
CALIB_SRCS = [os.path.join(HERE, "profiling", f) for f in ("calibrate.hip", "attention_loop.hip")]
CALIB_LIB = os.path.join(HERE, "profiling", "libaif_calib.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-result"]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _newest_header() -> float:
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    inc = os.path.join(HERE, "..", "include")
    hs += [os.path.join(inc, f) for f in os.listdir(inc) if f.endswith(".h")]
    return max(os.path.getmtime(h) for h in hs)


def _compile(src: str, force: bool) -> str:
    s = os.path.join(CSRC, src)
    o = os.path.join(OBJ, src[:-4] + ".o")
    dep = max(os.path.getmtime(s), _newest_header())
    if force or not os.path.exists(o) or os.path.getmtime(o) < dep:
        r = subprocess.run([HIPCC, *FLAGS, "-c", s, "-o", o], capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if err.strip():
            sys.stderr.write(err + "\n")
    return o


def build(force: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(sources()))) as ex:
        objs = list(ex.map(lambda f: _compile(f, force), sources()))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    if force or not os.path.exists(CALIB_LIB) or os.path.getmtime(CALIB_LIB) < max(os.path.getmtime(f) for f in CALIB_SRCS):
        r = subprocess.run([HIPCC, *FLAGS, "-shared", *CALIB_SRCS, "-o", CALIB_LIB], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on the calibration sources:\n" + "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l))
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
