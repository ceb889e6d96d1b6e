"""Compile the CPU oracle (plain C) into oracle/liblutnn_oracle.so.

Test infrastructure only; see the header of lutnn_oracle.c.

    python oracle/build.py [--sanitize]

--sanitize builds oracle/liblutnn_oracle_san.so instead: the same source under AddressSanitizer and
UndefinedBehaviorSanitizer (out-of-bounds accesses, signed overflow, misaligned or invalid
conversions abort with a report).  oracle/__init__.py loads that build when LUTNN_ORACLE_SANITIZE=1;
a Python process that loads it needs the ASan runtime preloaded (sanitizer_env() gives the
environment), which is how tests/test_oracle_sanitized.py runs the oracle's pins under it.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "lutnn_oracle.c")
LIB = os.path.join(HERE, "liblutnn_oracle.so")
LIB_SAN = os.path.join(HERE, "liblutnn_oracle_san.so")

# -ffp-contract=off: the only fused operations are the explicit fmaf() calls.
COMMON = ["-ffp-contract=off", "-fopenmp", "-fvisibility=hidden", "-shared", "-fPIC", "-Wall", "-Wextra"]
CMD = ["gcc", "-O2"] + COMMON + ["-o", LIB, SRC, "-lm"]
CMD_SAN = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all"] + COMMON + ["-o", LIB_SAN, SRC, "-lm"]


def build(force=True, sanitize=False):
    lib, cmd = (LIB_SAN, CMD_SAN) if sanitize else (LIB, CMD)
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC):
        return lib
    subprocess.run(cmd, check=True)
    return lib


def sanitizer_env(base=None):
    """Environment for a child Python process that is to load the sanitised build: the ASan runtime
    preloaded behind whatever is preloaded already, leak checking off (the interpreter is not
    instrumented), first error fatal."""
    env = dict(os.environ if base is None else base)
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True,
                          check=True).stdout.strip()
    env["LD_PRELOAD"] = ":".join(x for x in (env.get("LD_PRELOAD", ""), asan) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:halt_on_error=1:exitcode=86"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:exitcode=87"
    env["LUTNN_ORACLE_SANITIZE"] = "1"
    return env


if __name__ == "__main__":
    print(build(force=True, sanitize="--sanitize" in sys.argv))
    sys.exit(0)
