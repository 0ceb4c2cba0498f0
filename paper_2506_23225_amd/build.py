"""Compile the HIP sources under csrc/ into ``paper_2506_23225_amd/libmglu.so`` for gfx950.

``python -m paper_2506_23225_amd.build`` or :func:`build`.  hipcc cross-compiles
without a GPU; the library stays in-tree so that it travels with the sources.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmglu.so")
# the heavy files first: the kernels are instantiated per element type in files of their own so that they compile side by side
SOURCES = ["mglu_stream_bf16.hip", "mglu_stream_f16.hip", "mglu_stream_f32.hip", "mglu_prefill_bf16.hip",
           "mglu_prefill_f16.hip", "mglu_routed.hip", "mglu_api.hip", "mglu_pack.hip", "mglu_stream.hip", "mglu_prefill.hip", "mglu_route.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
    "-Wno-unused-command-line-argument",
    # packed-fp32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # leading kernel arguments arrive in scalar registers instead of being loaded by the kernel
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _deps_mtime():
    files = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    files.append(os.path.join(os.path.dirname(HERE), "include", "mglu.h"))
    return max(os.path.getmtime(f) for f in files)


def build(force=True, verbose=False, extra_flags=(), lib=LIB, obj_dir=OBJ):
    """Compile every source and link libmglu.so; with force=False only if it is absent or stale.

    `extra_flags` (e.g. -DMGLU_... tuning macros) together with another `lib` / `obj_dir`
    give a side build for experiments; the default arguments build the product."""
    sources = [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= _deps_mtime():
        return lib
    os.makedirs(obj_dir, exist_ok=True)
    hipcc = _hipcc()

    def compile_one(src):
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, res.stderr))
        if verbose and res.stderr:
            print(res.stderr, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 4)) as pool:
        objs = list(pool.map(compile_one, sources))
    tmp = lib + ".tmp.%d" % os.getpid()
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n%s" % res.stderr)
    os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
