"""Compile the HIP library for gfx950 (in-tree: paper_2603_09215_amd/libspark.so)."""
from __future__ import annotations

import pathlib
import subprocess

HERE = pathlib.Path(__file__).resolve().parent
CSRC = HERE / "csrc"
LIB = HERE / "libspark.so"

HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
               # packed fp32 instructions stay off for every HIP source of this library
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources() -> list[pathlib.Path]:
    return sorted(CSRC.glob("*.hip"))


def is_stale() -> bool:
    if not LIB.exists():
        return True
    t = LIB.stat().st_mtime
    deps = list(CSRC.glob("*")) + [HERE.parent / "include" / "spark.h"]
    return any(p.stat().st_mtime > t for p in deps)


def build(force: bool = True) -> pathlib.Path:
    if not force and not is_stale():
        return LIB
    cmd = ["hipcc", *HIPCC_FLAGS, "-o", str(LIB), *map(str, sources())]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stderr[-4000:])
    return LIB


if __name__ == "__main__":
    print("built", build())
