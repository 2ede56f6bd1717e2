"""Compile the C oracle into two shared libraries (fp32 arithmetic and its fp64 twin).

Test infrastructure: building the checker is not using it.  Run as a script or call build().
"""
from __future__ import annotations

import pathlib
import subprocess

HERE = pathlib.Path(__file__).resolve().parent
SRC = HERE / "spark_oracle.c"
LIBS = {"f32": HERE / "liboracle_f32.so", "f64": HERE / "liboracle_f64.so"}


def build(force: bool = True) -> None:
    for kind, out in LIBS.items():
        if not force and out.exists() and out.stat().st_mtime >= SRC.stat().st_mtime:
            continue
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra"]
        if kind == "f64":
            cmd.append("-DORA_REAL=double")
        cmd += ["-o", str(out), str(SRC), "-lm"]
        subprocess.run(cmd, check=True)


if __name__ == "__main__":
    build()
    print("built", ", ".join(str(p) for p in LIBS.values()))
