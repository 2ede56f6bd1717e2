"""Compile the HIP library for gfx950 (in-tree: paper_2603_09215_amd/libspark.so)."""
from __future__ import annotations

import pathlib
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = pathlib.Path(__file__).resolve().parent
CSRC = HERE / "csrc"
LIB = HERE / "libspark.so"

OBJ_DIR = HERE / "_build"

HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
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


def _compile(src: pathlib.Path) -> pathlib.Path:
    obj = OBJ_DIR / (src.stem + ".o")
    cmd = ["hipcc", *HIPCC_FLAGS, "-c", "-o", str(obj), str(src)]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src.name}:\n" + proc.stderr[-4000:])
    return obj


def build(force: bool = True, jobs: int = 8) -> pathlib.Path:
    """Compile every .hip translation unit (in parallel) and link them into libspark.so."""
    if not force and not is_stale():
        return LIB
    OBJ_DIR.mkdir(exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, sources()))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(LIB), *map(str, objs)]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("link failed:\n" + proc.stderr[-4000:])
    return LIB


if __name__ == "__main__":
    print("built", build())
