"""Build the gfx950 shared library (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libattnqat.so")
SOURCES = ["prep.hip", "fwd.hip", "bwd.hip", "mx.hip", "decode.hip", "api.hip"]
# bench-only helper with its own library: measurement code stays out of the attention library and its ABI
AUX_SRC = os.path.join(HERE, "benchaux", "mfma_burn.hip")
AUX_LIB = os.path.join(HERE, "benchaux", "libattnqat_benchaux.so")
# -packed-fp32-ops off: plain fp32 VALU code only (packed fp32 forms are not trusted here)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # one lane's atomic add stays one atomic add: the wave-wide rewrite of atomics makes the wave wait for the returned
         # value at once, which the decode kernel's ticket prefetch exists to avoid
         "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
         "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option", "-Wno-option-ignored"]


def _stale(out, deps):
    return not os.path.exists(out) or any(os.path.getmtime(d) > os.path.getmtime(out) for d in deps)


def build(force: bool = False, verbose: bool = False, extra=()) -> str:
    os.makedirs(OBJ, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hpp")]
    headers.append(os.path.join(os.path.dirname(HERE), "include", "attnqat.h"))

    def compile_one(src):
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ, src.replace(".hip", ".o"))
        if force or _stale(o, [s] + headers):
            cmd = ["hipcc", *FLAGS, *extra, "-c", s, "-o", o]
            if verbose:
                print(" ".join(cmd), flush=True)
            r = subprocess.run(cmd, capture_output=True, text=True)
            err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
            if r.returncode != 0:
                raise RuntimeError(f"hipcc failed on {src}:\n{err}")
            if verbose and err.strip():
                print(err)
        return o

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    if force or _stale(LIB, objs):
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    if force or _stale(AUX_LIB, [AUX_SRC]):
        r = subprocess.run(["hipcc", *FLAGS, "-shared", AUX_SRC, "-o", AUX_LIB], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {AUX_SRC}:\n{r.stderr}")
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
