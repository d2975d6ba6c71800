"""Compile the C oracle into oracle/liblorann_oracle.so (plain gcc, OpenMP over queries, no intrinsics)."""
from __future__ import annotations

import pathlib
import subprocess

HERE = pathlib.Path(__file__).resolve().parent
SRC = HERE / "lorann_oracle.c"
LIB = HERE / "liblorann_oracle.so"


def build(force: bool = True) -> pathlib.Path:
    if force or not LIB.exists() or LIB.stat().st_mtime < SRC.stat().st_mtime:
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", str(LIB), str(SRC), "-lm"]
        subprocess.run(cmd, check=True)
    return LIB


SAN_LIB = HERE / "liblorann_oracle_san.so"


def build_sanitized() -> pathlib.Path:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (any report ends the process).  Loading
    it into Python needs gcc's libasan first in the process (sanitizer_runtime()); LORANN_ORACLE_LIB=<path> makes
    oracle.lib() load it instead of the plain build."""
    cmd = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", str(SAN_LIB), str(SRC), "-lm"]
    subprocess.run(cmd, check=True)
    return SAN_LIB


def sanitizer_runtime() -> str:
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()


if __name__ == "__main__":
    print(build())
