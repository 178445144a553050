"""Compile the C oracle into oracle/libpasgd_oracle.so (gcc, no fast-math), and the same source
with fp32 accumulators into oracle/libpasgd_oracle_f32acc.so (a sensitivity probe for tests)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "pasgd_oracle.c")
LIB = os.path.join(HERE, "libpasgd_oracle.so")
LIB_F32ACC = os.path.join(HERE, "libpasgd_oracle_f32acc.so")


def _fresh(lib: str) -> bool:
    return os.path.exists(lib) and os.path.getmtime(lib) >= max(
        os.path.getmtime(SRC), os.path.getmtime(os.path.join(HERE, "pasgd_oracle.h")))


def build(force: bool = True) -> str:
    for lib, defs in ((LIB, []), (LIB_F32ACC, ["-DORC_ACC_FLOAT"])):
        if not force and _fresh(lib):
            continue
        cmd = ["gcc", "-O2", "-std=c11", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-fPIC",
               "-shared", "-Wall", "-Wextra", *defs, "-o", lib, SRC, "-lm"]
        subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build())
