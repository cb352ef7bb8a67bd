"""Compiles the CPU oracle (plain C) into oracle/liboracle.so with gcc.

The oracle is test infrastructure; building it is not using it.
-ffp-contract=off keeps every fp32/fp64 operation a separately rounded one,
which the canonical distance relies on.

A sanitizer leg for the CPU side of the repository:

    TSDG_ORACLE_SANITIZE=1 ASAN_OPTIONS=detect_leaks=0 \\
    LD_PRELOAD="$(gcc -print-file-name=libasan.so) $(gcc -print-file-name=libubsan.so)${LD_PRELOAD:+ $LD_PRELOAD}" \\
        python -m pytest tests -m "not gpu" -p no:cacheprovider

builds oracle/liboracle_san.so with -fsanitize=address,undefined (-O1 -g, no recovery from undefined
behaviour) and loads that instead; the preload puts the sanitizer runtimes ahead of python's own
allocator, which a sanitized shared object inside an unsanitized interpreter needs.  `python -m
oracle.build --sanitize` only compiles it.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "tsdg_oracle.c")
OUT = os.path.join(HERE, "liboracle.so")
OUT_SAN = os.path.join(HERE, "liboracle_san.so")
COMMON = ["-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra"]


def sanitize_requested() -> bool:
    return os.environ.get("TSDG_ORACLE_SANITIZE", "") == "1"


def build(force: bool = True, sanitize: bool = None) -> str:
    if sanitize is None:
        sanitize = sanitize_requested()
    out = OUT_SAN if sanitize else OUT
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
        return out
    opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer"] if sanitize else ["-O2"]
    subprocess.run(["gcc", *opt, *COMMON, "-o", out, SRC, "-lm"], check=True)
    return out


if __name__ == "__main__":
    print(build(force=True, sanitize="--sanitize" in sys.argv or sanitize_requested()))
    sys.exit(0)
