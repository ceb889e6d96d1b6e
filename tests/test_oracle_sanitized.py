"""The oracle's pins once more, with the C oracle compiled under AddressSanitizer and
UndefinedBehaviorSanitizer (oracle/build.py --sanitize): an out-of-bounds read or write, a signed
overflow or an invalid conversion anywhere in the plain loops that every parity claim rests on ends
the child process with a report.  CPU only."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = ["tests/test_oracle_encode.py", "tests/test_oracle_table_lookup.py", "tests/test_oracle_tree.py"]


def test_oracle_pins_pass_under_asan_and_ubsan():
    sys.path.insert(0, ROOT)
    from oracle import build
    lib = build.build(force=True, sanitize=True)
    syms = subprocess.run(["nm", "-D", lib], capture_output=True, text=True, check=True).stdout
    assert "__asan_init" in syms and "__ubsan_handle" in syms, "the sanitised build is not instrumented"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + PINS,
                       cwd=ROOT, env=build.sanitizer_env(), capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-4000:]
    assert "AddressSanitizer" not in tail and "runtime error" not in tail, tail
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "failed" not in r.stdout, tail
    # the child really loaded the sanitised library
    probe = ("import oracle, os; oracle.threads(); "
             "print(any('liblutnn_oracle_san' in l for l in open('/proc/self/maps')))")
    r = subprocess.run([sys.executable, "-c", probe], cwd=ROOT, env=build.sanitizer_env(), capture_output=True,
                       text=True, timeout=300)
    assert r.stdout.strip() == "True", r.stdout + r.stderr


def test_the_sanitizer_is_live():
    """A child process hands the sanitised oracle an index buffer that is too small (the mistake is
    planted in the call, on the CPU): the first write past its end must end the child with ASan's
    report and exit code, not with wrong memory."""
    sys.path.insert(0, ROOT)
    from oracle import build
    build.build(force=False, sanitize=True)
    code = (
        "import numpy as np, ctypes, oracle\n"
        "lib = oracle._lib()\n"
        "P = np.zeros((2, 16, 4), np.float32); X = np.zeros((64, 8), np.float32)\n"
        "idx = np.zeros(10, np.uint8)  # 64 rows x 2 codebooks need 128 bytes\n"
        "f, u = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_uint8)\n"
        "lib.lutnn_oracle_encode(P.ctypes.data_as(f), 2, 16, 4, X.ctypes.data_as(f), 64, 8, idx.ctypes.data_as(u))\n"
        "print('survived')\n")
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=build.sanitizer_env(), capture_output=True,
                       text=True, timeout=300)
    assert r.returncode == 86 and "heap-buffer-overflow" in r.stderr and "survived" not in r.stdout, \
        (r.returncode, r.stderr[-800:])
