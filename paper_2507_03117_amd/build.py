"""Build the HIP library for gfx950 in-tree: paper_2507_03117_amd/libblast_hip.so."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libblast_hip.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
    "-munsafe-fp-atomics",
    # packed-fp32 instruction selection stays off on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = False) -> str:
    """Compiles every csrc/*.hip (one hipcc process per file, side by side) and links the shared library."""
    from concurrent.futures import ThreadPoolExecutor

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in HIPCC_FLAGS if f != "-shared"]

    def filtered(res):
        # the host pass prints a harmless note that it does not know the packed-fp32 feature
        return "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)

    def compile_one(src):
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        res = subprocess.run([hipcc] + compile_flags + ["-c", src, "-o", obj], capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, filtered(res)))
        return obj, filtered(res)

    with ThreadPoolExecutor(max_workers=min(8, len(sources()))) as pool:
        done = list(pool.map(compile_one, sources()))
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc"] + [o for o, _ in done] +
                         ["-o", LIB + ".tmp"], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + filtered(res))
    os.replace(LIB + ".tmp", LIB)
    if verbose:
        for _, err in done:
            if err.strip():
                print(err)
    return LIB


def stale() -> bool:
    """True when the library is missing or older than any of the sources it is built from."""
    if not os.path.exists(LIB):
        return True
    built = os.path.getmtime(LIB)
    deps = glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.h")) + \
        glob.glob(os.path.join(os.path.dirname(HERE), "include", "*.h"))
    return any(os.path.getmtime(d) > built for d in deps)


def ensure_built() -> str:
    """Build if no library is there or a source is newer than it (tests, the smoke check and the benchmark call
    this; the binding itself never builds and raises when the library is missing).  Where no compiler is
    installed a library that is there is used as it is."""
    if not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if os.path.exists(LIB) and not os.path.exists(hipcc):
        return LIB
    return build()


if __name__ == "__main__":
    print(build(verbose=True))
