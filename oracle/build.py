"""Builds the CPU oracle (test infrastructure) into oracle/libg10_oracle.so.

With G10_ORACLE_SANITIZE=1 in the environment (or `--sanitize`) the library is built with
AddressSanitizer and UndefinedBehaviorSanitizer into oracle/libg10_oracle_san.so instead, and
that is what oracle.py then loads.  A sanitized shared library needs the sanitizer runtime in
the process first; run the CPU tests under it as

    G10_ORACLE_SANITIZE=1 LD_PRELOAD=$(gcc -print-file-name=libasan.so) \\
        ASAN_OPTIONS=detect_leaks=0 python -m pytest tests -q -m "not gpu"

(leak detection off: the Python interpreter itself never frees everything).
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "g10_oracle.cpp")
LIB = os.path.join(HERE, "libg10_oracle.so")
LIB_SAN = os.path.join(HERE, "libg10_oracle_san.so")


def sanitize_wanted() -> bool:
    return os.environ.get("G10_ORACLE_SANITIZE", "") not in ("", "0")


def build(force: bool = False, sanitize=None) -> str:
    if sanitize is None:
        sanitize = sanitize_wanted()
    lib = LIB_SAN if sanitize else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC):
        return lib
    flags = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"] if sanitize else ["-O2"]
    cmd = ["g++", "-std=c++17"] + flags + ["-Wall", "-Wextra", "-shared", "-fPIC", SRC, "-o", lib]
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, sanitize=True if "--sanitize" in sys.argv else None))
