"""Build step of the HIP library: hipcc cross-compiles every source under
``csrc/`` for gfx950 into ``libmoe_hip.so`` next to this file (in-tree, so the
built library travels with the source tree)."""
import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_hip.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build_hip(verbose=False, defines=(), out=None):
    """Compile and link the library.  ``defines`` (e.g. ["MOE_STREAM_SWIZZLE_A=0"]) and ``out`` build a variant
    for layout studies into another file; the default call builds the product next to this module."""
    csrc = os.path.join(_HERE, "csrc")
    obj_dir = os.path.join(_HERE, "_build" if not defines else "_build_" + "_".join(d.replace("=", "") for d in defines))
    lib_path = out or LIB_PATH
    os.makedirs(obj_dir, exist_ok=True)
    sources = sorted(glob.glob(os.path.join(csrc, "*.hip")))
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

    def compile_one(src):
        obj = os.path.join(obj_dir, os.path.basename(src) + ".o")
        cmd = [hipcc] + HIPCC_FLAGS + ["-D" + d for d in defines] + ["-c", src, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, r.stderr))
        if verbose and r.stderr.strip():
            print(r.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(sources))) as ex:
        objs = list(ex.map(compile_one, sources))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib_path] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s" % r.stderr)
    return lib_path


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser(description=__doc__)
    ap.add_argument("--define", action="append", default=[], help="NAME=VALUE passed to hipcc as -D (layout-study switches)")
    ap.add_argument("--out", default=None, help="output file of a variant build (default: the product library)")
    a = ap.parse_args()
    if a.define and not a.out:
        ap.error("a build with --define is a study variant: give it its own --out file")
    print(build_hip(verbose=True, defines=a.define, out=a.out))
