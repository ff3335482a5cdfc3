"""Builds libevconv.so (HIP kernels + C ABI) for gfx950, in-tree, with hipcc.

Every csrc/*.hip is compiled to an object file of its own (in parallel) and the objects are
linked into the shared library.  build() recompiles everything; build(incremental=True) only
what is older than its source or than a header (development loop).
"""
import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libevconv.so")
PHASE_LIB_PATH = os.path.join(_HERE, "libevconv_phase_stamps.so")  # the build with -DEVCONV_PHASE_STAMPS
OBJ_DIR = os.path.join(_HERE, "_build")

# Packed-fp32 VALU instructions are switched off for every device translation unit.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-bitwise-instead-of-logical",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = False, incremental: bool = False, jobs: int = 8, phase_stamps: bool = False) -> str:
    """phase_stamps: the measurement build whose matrix-core kernels record per-phase time stamps
    (evconv_debug_phase_stamps); it goes to a library of its own and leaves libevconv.so alone."""
    srcs = sorted(glob.glob(os.path.join(_HERE, "csrc", "*.hip")))
    headers = glob.glob(os.path.join(_HERE, "csrc", "*.h")) + glob.glob(os.path.join(_HERE, "..", "include", "*.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    obj_dir = OBJ_DIR + ("_phase_stamps" if phase_stamps else "")
    flags = HIPCC_FLAGS + (["-DEVCONV_PHASE_STAMPS"] if phase_stamps else [])
    lib_path = PHASE_LIB_PATH if phase_stamps else LIB_PATH
    os.makedirs(obj_dir, exist_ok=True)
    objs = [os.path.join(obj_dir, os.path.basename(s)[:-4] + ".o") for s in srcs]

    def compile_one(pair):
        src, obj = pair
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
            return
        cmd = [hipcc] + flags + ["-c", "-o", obj, src]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        # (the host pass does not know the packed-fp32 feature and says so once per file: harmless)
        text = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
        if text.strip():
            print(text, file=sys.stderr, flush=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}")

    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(srcs)))) as pool:
        list(pool.map(compile_one, zip(srcs, objs)))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib_path] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return lib_path


if __name__ == "__main__":
    build(verbose=True, incremental="--incremental" in sys.argv, phase_stamps="--phase-stamps" in sys.argv)
