"""Compile the C part of the oracle with gcc (test infrastructure; never used by the product path)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
BUILD = os.path.join(HERE, "_build")
SRC = os.path.join(HERE, "branch_attention.c")


def lib_path(real: str = "f64") -> str:
    return os.path.join(BUILD, f"liboracle_{real}.so")


def build(force: bool = False) -> None:
    os.makedirs(BUILD, exist_ok=True)
    for real, ctype in (("f64", "double"), ("f32", "float")):
        out = lib_path(real)
        if (not force and os.path.exists(out)
                and os.path.getmtime(out) >= os.path.getmtime(SRC)):
            continue
        cmd = ["gcc", "-O2", "-march=x86-64-v3", "-fopenmp", "-std=c99", "-Wall", "-Wextra",
               "-fno-fast-math", f"-DORACLE_REAL={ctype}", "-shared", "-fPIC", "-o", out, SRC, "-lm"]
        subprocess.run(cmd, check=True)


if __name__ == "__main__":
    build(force=True)
    print("built", lib_path("f64"), lib_path("f32"))
