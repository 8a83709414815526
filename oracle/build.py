"""Compile the C oracle with gcc.

build()            oracle/libmoe_oracle.so: generic x86-64, -O2, OpenMP: the checker every test uses.
build_native()     oracle/libmoe_oracle_native.so: the same source with -O3 -march=native, for the
                   benchmark's CPU-baseline leg only (it is timed, never used as a reference:
                   -march=native may contract multiply-adds, which changes last bits).
build_sanitized()  an AddressSanitizer + UndefinedBehaviorSanitizer build of a C driver that includes
                   the oracle's source and walks every function over ragged shapes (tests/sanitize_oracle.c).
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "moe_oracle.c")
LIB = os.path.join(HERE, "libmoe_oracle.so")
LIB_NATIVE = os.path.join(HERE, "libmoe_oracle_native.so")
COMMON = ["gcc", "-std=c99", "-fopenmp", "-Wall", "-Wextra"]


def build(force: bool = True, src: str = SRC, out: str = LIB) -> str:
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(src):
        return out
    subprocess.run([*COMMON, "-O2", "-shared", "-fPIC", src, "-o", out, "-lm"], check=True)
    return out


def build_native(out: str = LIB_NATIVE) -> str:
    subprocess.run([*COMMON, "-O3", "-march=native", "-shared", "-fPIC", SRC, "-o", out, "-lm"], check=True)
    return out


def build_sanitized(driver_src: str, out: str) -> str:
    """Executable with the sanitizer runtimes linked in statically (no preloading needed)."""
    subprocess.run([*COMMON, "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=undefined", "-static-libasan", "-static-libubsan",
                    "-I", HERE, driver_src, "-o", out, "-lm"], check=True)
    return out


if __name__ == "__main__":
    print(build())
