"""Build libcat_hip.so (gfx950) in-tree with hipcc.

    python -m paper_2509_26277_amd.build [--force]

hipcc cross-compiles without a GPU.  Packed-FP32 instruction selection is switched
off for all device code, and floating-point atomics are allowed to use the native
LDS / L2 add instructions.
"""
import os
import subprocess
import sys
import time

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
# (the files that take longest to compile come first: they start at once and the rest fills in beside them)
SOURCES = ["cat_tile_k16_f32.hip", "cat_tile_k16_bf16.hip", "cat_tile_k16_f32_p1.hip", "cat_tile_k16_bf16_p1.hip",
           "cat_tile_bounds_f32.hip", "cat_tile_bounds_bf16.hip", "cat_infer.hip", "cat_api.hip", "cat_stream.hip", "cat_tile.hip",
           "cat_pca.hip", "cat_sweep.hip", "cat_seed.hip", "cat_lds.hip", "cat_lp.hip", "cat_tile_multi_f32.hip",
           "cat_tile_multi_bf16.hip", "cat_tile_split.hip"] + [
    f"cat_tile_k{kt}_{dt}.hip" for kt in (8, 4, 2, 1) for dt in ("f32", "bf16")]
HEADERS = ["cat_common.h", "cat_tile.h", "cat_tile_kernel.h", "cat_infer.h", "cat_infer_kernel.h"]
OUT = os.path.join(_HERE, "libcat_hip.so")
OBJ_DIR = os.path.join(_HERE, "_build")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-munsafe-fp-atomics",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(_ROOT, "include"), "-I", CSRC,
]


def _newer(a, b):
    return not os.path.exists(b) or os.path.getmtime(a) > os.path.getmtime(b)


def build(force=False, verbose=True):
    os.makedirs(OBJ_DIR, exist_ok=True)
    deps = [os.path.join(CSRC, h) for h in HEADERS] + [os.path.join(_ROOT, "include", "cat.h"), __file__]
    objs, procs = [], []
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        objs.append(o)
        if force or _newer(s, o) or any(_newer(d, o) for d in deps):
            cmd = ["hipcc", "-c", *FLAGS, "-o", o, s]
            if verbose:
                print(" ".join(cmd), flush=True)
            while sum(p.poll() is None for _, p in procs) >= max(2, (os.cpu_count() or 4)):
                time.sleep(0.2)
            procs.append((src, subprocess.Popen(cmd)))
    for src, p in procs:
        if p.wait() != 0:
            raise RuntimeError(f"hipcc failed on {src}")
    if force or procs or not os.path.exists(OUT):
        cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT, *objs]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    build(force="--force" in sys.argv)
    print(OUT)
