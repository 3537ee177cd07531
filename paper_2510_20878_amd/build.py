"""Compile csrc/ for gfx950 into lib/libha_rag.so with hipcc (works without a GPU)."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIBDIR = os.path.join(HERE, "lib")
LIB = os.path.join(LIBDIR, "libha_rag.so")
SOURCES = ["ha_rag_kernels.hip", "ha_rag_attend_kernels.hip", "ha_rag_attend_shared.hip", "ha_rag_api.hip", "ha_rag_pool.hip",
           "ha_rag_load.hip", "ha_rag_attend.hip", "ha_rag_io.hip"]
HEADERS = [os.path.join(CSRC, "ha_rag_kernels.h"), os.path.join(CSRC, "ha_rag_internal.h"),
           os.path.join(CSRC, "ha_rag_decode.h"), os.path.join(CSRC, "ha_rag_attend_dev.h"),
           os.path.join(os.path.dirname(HERE), "include", "ha_rag.h")]

# Packed fp32 instructions are switched off for every device compilation.  Inputs are finite
# by contract, so min/max need not quiet signalling NaNs first (-fno-honor-nans); nothing else
# of fast-math is enabled: divisions, fmas and conversions keep their IEEE results.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
               "-ffp-contract=off",
               "-fno-fast-math", "-fno-honor-nans", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops",
               "-Wall", "-Wno-unused-command-line-argument"]


def up_to_date() -> bool:
    if not os.path.exists(LIB):
        return False
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return all(os.path.getmtime(d) <= t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and up_to_date():
        return LIB
    os.makedirs(LIBDIR, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        hipcc = "hipcc"
    # one hipcc per source, side by side; then one link.  Every call compiles every source.
    objdir = os.path.join(LIBDIR, "_build")
    os.makedirs(objdir, exist_ok=True)
    noise = ("packed-fp32-ops", "is not a recognized feature")

    def compile_one(src):
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc] + HIPCC_FLAGS + ["-c", "-o", obj, os.path.join(CSRC, src)]
        if verbose:
            print(" ".join(cmd))
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if not any(n in l for n in noise))
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on " + src + ":\n" + err)
        return obj, err

    jobs = max(1, min(len(SOURCES), os.cpu_count() or 1, int(os.environ.get("MAX_JOBS", "16"))))
    with ThreadPoolExecutor(jobs) as pool:
        done = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + [o for o, _ in done]
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc link failed:\n" + r.stderr)
    err = "\n".join(e for _, e in done if e.strip())
    if verbose and err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
