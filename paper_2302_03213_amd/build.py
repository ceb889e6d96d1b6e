"""Compile liblutnn.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2302_03213_amd.build

Objects go to _build/ at the repository root (not committed); the shared library is written
next to this file so that it travels with the source tree.
"""
import concurrent.futures
import hashlib
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
OBJDIR = os.path.join(ROOT, "_build")
LIB = os.path.join(PKG, "liblutnn.so")

SOURCES = ["api.hip", "encode.hip", "encode_tree.hip", "build_table.hip", "lookup_lds.hip", "lookup_rows.hip", "lookup_mfma.hip", "lookup_smfmac.hip", "lookup_wide.hip",
           "linear_fused.hip", "linear_small.hip", "softpq_backward.hip", "probe_smfmac.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# packed-fp32 VALU ops are switched off for every device compile in this project.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function",
         # the LDS-direct loads set M0 in inline assembly and name it as clobbered; clang warns on every
         # instantiation that M0 is a reserved register (it is not live across those statements)
         "-Wno-inline-asm", "-I", INCLUDE, "-I", CSRC]


def source_hash():
    """12 hex digits over every file the library is compiled from (csrc/*, include/lutnn.h); the
    library reports it through lutnn_version() so that the loader can tell a stale binary."""
    h = hashlib.sha256()
    files = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith((".hip", ".h"))]
    for path in files + headers():
        h.update(os.path.basename(path).encode() + b"\0")
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:12]


def _compile(src):
    obj = os.path.join(OBJDIR, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    if src == "api.hip":
        cmd.append('-DLUTNN_SOURCE_HASH="%s"' % source_hash())
    r = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                    if "packed-fp32-ops" not in l)  # host pass does not know the device feature
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, out))
    return obj, out


def build(verbose=False):
    os.makedirs(OBJDIR, exist_ok=True)
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
    print(build(verbose=True))
