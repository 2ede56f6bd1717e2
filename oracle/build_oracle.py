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


def build_sanitized(kind: str = "f32") -> pathlib.Path:
    """The oracle with AddressSanitizer and UndefinedBehaviorSanitizer (host code only), linked
    with a driver that walks every entry point on a tiny model (sanitize_check.c).  The runtime is
    linked statically so that the program does not depend on library preload order."""
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-static-libasan", "-Wall", "-Wextra",
           "-o", str(HERE / f"sanitize_check_{kind}"), str(HERE / "sanitize_check.c"), "-lm"]
    if kind == "f64":
        cmd.insert(1, "-DORA_REAL=double")
    subprocess.run(cmd, check=True)
    return HERE / f"sanitize_check_{kind}"


def run_sanitized(kind: str = "f32", threads: int = 4) -> subprocess.CompletedProcess:
    """build and run the sanitized driver for one arithmetic type"""
    import os
    env = dict(os.environ, OMP_NUM_THREADS=str(threads), ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    exe = build_sanitized(kind)
    return subprocess.run([str(exe)], env=env, capture_output=True, text=True, timeout=600)


if __name__ == "__main__":
    build()
    print("built", ", ".join(str(p) for p in LIBS.values()))
