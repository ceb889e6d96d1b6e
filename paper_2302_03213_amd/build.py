"""Compile liblutnn.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2302_03213_amd.build

Objects go to _build/ at the repository root (not committed); the shared library is written
next to this file so that it travels with the source tree.
"""
import concurrent.futures
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
OBJDIR = os.path.join(ROOT, "_build")
LIB = os.path.join(PKG, "liblutnn.so")

SOURCES = ["api.hip", "encode.hip", "encode_tree.hip", "build_table.hip", "lookup_lds.hip", "lookup_rows.hip", "lookup_mfma.hip", "lookup_smfmac.hip",
           "linear_fused.hip", "linear_small.hip", "softpq_backward.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# packed-fp32 VALU ops are switched off for every device compile in this project.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-I", INCLUDE, "-I", CSRC]


def _compile(src):
    obj = os.path.join(OBJDIR, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                    if "packed-fp32-ops" not in l)  # host pass does not know the device feature
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, out))
    return obj, out


def build(verbose=False, save_temps=False):
    os.makedirs(OBJDIR, exist_ok=True)
    if save_temps:
        FLAGS.extend(["-save-temps=obj"])
    with concurrent.futures.ThreadPoolExecutor(max_workers=6) as ex:
        results = list(ex.map(_compile, SOURCES))
    if verbose:
        for _, out in results:
            if out.strip():
                print(out)
    objs = [o for o, _ in results]
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.run(cmd, check=True)
    return LIB


def headers():
    return [os.path.join(INCLUDE, "lutnn.h")]


if __name__ == "__main__":
    print(build(verbose=True, save_temps="--save-temps" in sys.argv))
