"""Compile the C oracle with gcc (no GPU involved): oracle/liboracle.so is the build every test
uses (-O2); oracle/liboracle_native.so is the same source at -O3 -march=native, which only the
benchmark's timed CPU-baseline leg loads (after checking that it agrees with the first)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "ha_rag_oracle.c")
LIB = os.path.join(HERE, "liboracle.so")
LIB_NATIVE = os.path.join(HERE, "liboracle_native.so")
COMMON = ["-std=c99", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-Wall", "-Wextra"]


def _fresh(lib):
    return os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC)


def build(force: bool = True) -> str:
    if not force and _fresh(LIB):
        return LIB
    subprocess.run(["gcc", "-O2"] + COMMON + ["-o", LIB, SRC, "-lm"], check=True)
    return LIB


def build_native(force: bool = True) -> str:
    """For the machine it runs on: built where it is timed."""
    if not force and _fresh(LIB_NATIVE):
        return LIB_NATIVE
    out = LIB_NATIVE
    if not os.access(HERE, os.W_OK):  # a read-only checkout: keep the build beside the temp files
        import tempfile
        out = os.path.join(tempfile.gettempdir(), "liboracle_native_%d.so" % os.getuid())
    subprocess.run(["gcc", "-O3", "-march=native"] + COMMON + ["-o", out, SRC, "-lm"], check=True)
    return out


if __name__ == "__main__":
    print(build())
