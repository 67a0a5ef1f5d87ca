"""Compile the C oracle into oracle/libmhffn_oracle.so with gcc.

Test infrastructure only.  Run as `python -m oracle.build` or through
`oracle.mhffn_oracle.load()` which builds when the library is missing."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "mhffn_oracle.c")
LIB = os.path.join(HERE, "libmhffn_oracle.so")

# x86-64-v3 (AVX2 + FMA) rather than -march=native: the built library is
# carried to another machine whose CPU may differ from the build host's.
CFLAGS = ["-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared",
          "-std=c11", "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and \
            os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, SRC, "-lm"])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
