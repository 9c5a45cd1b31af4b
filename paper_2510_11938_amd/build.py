"""Build the HIP library in-tree: one hipcc compile per translation unit, then a
shared link.  ``python -m paper_2510_11938_amd.build`` or ``build.build()``."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libflexstage.so")
UNITS = ["flexstage", "kv_move", "weight_pack", "gemm_skinny", "gemm_tiled", "epilogue", "attn_decode", "attn_prefill",
         "granularity"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# Per-unit additions.  attn_prefill: matrix-core results stay in ordinary vector registers; with the default choice the
# compiler kept the output accumulators in vector registers between tiles and copied all 32 of them to accumulation
# registers and back around the products of every tile (64 moves per tile and wavefront in a loop bound by vector ALU work).
UNIT_FLAGS = {"attn_prefill": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def _stale(target: str, deps) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, verbose: bool = False, tuning: bool = False) -> str:
    """tuning=True builds libflexstage_tuning.so instead: the same sources with -DFXP_TUNING, whose launch shapes can be
    overridden through FXP_* environment variables (kernel experiments only; the normal build ignores them)."""
    global OBJ, LIB
    if tuning:
        OBJ, LIB = os.path.join(HERE, "_build_tuning"), os.path.join(HERE, "libflexstage_tuning.so")
    os.makedirs(OBJ, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers.append(os.path.join(os.path.dirname(HERE), "include", "flexstage.h"))

    def compile_one(u: str) -> str:
        src, obj = os.path.join(CSRC, u + ".hip"), os.path.join(OBJ, u + ".o")
        if force or _stale(obj, [src] + headers):
            r = subprocess.run(["hipcc", *FLAGS, *(["-DFXP_TUNING"] if tuning else []), *UNIT_FLAGS.get(u, []), "-c", src, "-o", obj],
                               capture_output=True, text=True)
            err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
            if r.returncode != 0:
                raise RuntimeError(f"hipcc failed on {u}.hip:\n{err}")
            if verbose and err.strip():
                print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(compile_one, UNITS))
    if force or _stale(LIB, objs):
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True, tuning="--tuning" in sys.argv))
