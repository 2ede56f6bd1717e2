"""Compile the HIP library for gfx950 (in-tree: paper_2603_09215_amd/libspark.so)."""
from __future__ import annotations

import pathlib
import re
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


def kernel_resources(remarks: str) -> dict[str, dict[str, int]]:
    """per kernel, the figures of the compiler's resource-usage remarks (registers, scratch bytes
    per lane, spills, waves per SIMD, LDS bytes)"""
    table: dict[str, dict[str, int]] = {}
    name = None
    for line in remarks.splitlines():
        m = re.search(r"remark: Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            table[name] = {}
            continue
        m = re.search(r"remark:\s+([A-Za-z][A-Za-z /\[\]]*?): (\d+) \[-Rpass-analysis", line)
        if m and name:
            table[name][m.group(1).strip()] = int(m.group(2))
    return table


def _compile(src: pathlib.Path) -> pathlib.Path:
    """One translation unit.  A kernel that uses scratch memory fails the build: every access to it
    is a memory round trip, and in these kernels it has only ever meant an array that the compiler
    could not keep in registers (an index computed at run time)."""
    obj = OBJ_DIR / (src.stem + ".o")
    cmd = ["hipcc", *HIPCC_FLAGS, "-Rpass-analysis=kernel-resource-usage", "-c", "-o", str(obj), str(src)]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src.name}:\n" + proc.stderr[-4000:])
    table = kernel_resources(proc.stderr)
    (OBJ_DIR / (src.stem + ".resources.txt")).write_text(
        "".join(f"{k} {' '.join(f'{a}={b}' for a, b in v.items())}\n" for k, v in sorted(table.items())))
    bad = [k for k, v in table.items() if v.get("ScratchSize [bytes/lane]", 0) or v.get("VGPRs Spill", 0)]
    if bad:
        raise RuntimeError(f"{src.name}: kernels with scratch memory or spilled registers:\n  " + "\n  ".join(bad))
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
