"""Compile the CPU oracle (plain C, FP64) into oracle/liboracle.so with gcc.

Test infrastructure only: the HIP library never links or loads this.
Run as ``python -m oracle.build`` or call ``build()``.

``build(sanitize=True)`` (``python -m oracle.build --sanitize``) makes a second library,
oracle/liboracle_san.so, compiled with AddressSanitizer and UndefinedBehaviorSanitizer (host code only,
``-fsanitize=address,undefined -O1 -g``).  The oracle loads that one when the environment variable
DMATH_ORACLE_SANITIZE is 1; the interpreter must then run with the sanitizer runtime preloaded:

    LD_PRELOAD=$(gcc -print-file-name=libasan.so) ASAN_OPTIONS=detect_leaks=0 DMATH_ORACLE_SANITIZE=1 \\
        python -m pytest tests/test_oracle_pins.py -q

(``tests/test_oracle_sanitized.py`` does exactly this in a child process.)
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "dmath_oracle.c")
LIB = os.path.join(HERE, "liboracle.so")
LIB_SANITIZED = os.path.join(HERE, "liboracle_san.so")
SANITIZE_FLAGS = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
                  "-O1", "-g"]


def sanitizer_runtime() -> str:
    """Path of the AddressSanitizer runtime that a process loading the sanitized oracle must preload."""
    return subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()


def build(force: bool = True, sanitize: bool = False) -> str:
    lib = LIB_SANITIZED if sanitize else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC):
        return lib
    tmp = lib + ".tmp.%d" % os.getpid()
    opt = SANITIZE_FLAGS if sanitize else ["-O2"]
    cmd = ["gcc"] + opt + ["-fopenmp", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", tmp, SRC, "-lm"]
    subprocess.check_call(cmd)
    os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    print(build(force=True, sanitize="--sanitize" in sys.argv))
    sys.exit(0)
