"""Build libosdn.so (the HIP library) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libosdn.so")
SOURCES = ["osdn_api.hip", "osdn_precond.hip", "osdn_precond_bwd.hip", "osdn_precond_gen.hip", "osdn_step.hip", "osdn_pad.hip",
           "osdn_chunk_fwd.hip", "osdn_chunk_bwd.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def build(verbose: bool = False, only=None) -> str:
    """Compile every HIP source of the library (side by side, one hipcc per file) and link
    them into one shared object.  `only`: recompile just these sources and reuse the other
    objects of an earlier build (for quick iteration; the default compiles everything)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)

    # an object is reused only if it is newer than every header (the kernels pass their arguments
    # in structs declared there: an object built against an older layout must never be linked)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers.append(os.path.join(os.path.dirname(HERE), "include", "osdn.h"))
    newest_header = max(os.path.getmtime(h) for h in headers if os.path.exists(h))

    def compile_one(src):
        obj = os.path.join(OBJ, src.replace(".hip", ".o"))
        if (only is not None and src not in only and os.path.exists(obj)
                and os.path.getmtime(obj) > max(newest_header, os.path.getmtime(os.path.join(CSRC, src)))):
            return obj
        cmd = [hipcc, *FLAGS, "-c", "-o", obj, os.path.join(CSRC, src)]
        if verbose:
            print(" ".join(cmd))
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0 or verbose:
            print(r.stdout)
        if r.returncode != 0:
            raise subprocess.CalledProcessError(r.returncode, cmd)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose=True, only=sys.argv[1:] or None))
