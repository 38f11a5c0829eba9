"""Build the CPU oracle (test infrastructure) into two shared libraries: float32 and float64 arithmetic."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "sjd_oracle.c")
FLAGS = ["-O3", "-std=gnu99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
         "-fvisibility=hidden", "-Wall", "-Wextra"]


def lib_path(real: str) -> str:
    return os.path.join(HERE, f"libsjd_oracle_{real}.so")


def build(force: bool = True) -> None:
    for real, ctype in (("f32", "float"), ("f64", "double")):
        out = lib_path(real)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
            continue
        cmd = ["gcc", *FLAGS, f"-DREAL={ctype}", SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


if __name__ == "__main__":
    build()
    print("built", lib_path("f32"), lib_path("f64"))
