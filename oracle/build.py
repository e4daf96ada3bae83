"""Compile the C oracle into oracle/libblast_oracle.so (gcc, OpenMP, no fast-math)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "blast_oracle.c")
LIB = os.path.join(HERE, "libblast_oracle.so")


def build(force: bool = False) -> str:
    # a test may point the front-end at another build of the same source (sanitizer build, planted mistake)
    override = os.environ.get("BLAST_ORACLE_LIB")
    if override and not force:
        return override
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-fast-math", "-Wall", "-Wextra",
           SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


def build_variant(out: str, source_text: str = None, sanitize: bool = False) -> str:
    """Compiles the oracle (or an edited copy of its source text) into `out`; with `sanitize`, under
    AddressSanitizer and UndefinedBehaviorSanitizer (the process that loads it must preload libasan)."""
    src = SRC
    if source_text is not None:
        src = out + ".c"
        with open(src, "w") as f:
            f.write(source_text)
    cmd = ["gcc", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-fast-math", "-Wall", "-Wextra"]
    cmd += ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"] \
        if sanitize else ["-O2"]
    subprocess.run(cmd + [src, "-o", out, "-lm"], check=True, capture_output=True)
    return out


if __name__ == "__main__":
    print(build(force=True))
